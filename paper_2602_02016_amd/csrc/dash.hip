// Host side of the C ABI declared in include/dash.h: argument checks, workspace
// carving, chunking of long stacks, and the launch sequences of the paper's methods.
// Every arithmetic step runs in the kernels of gemm.hip / elementwise.hip.
#include "../../include/dash.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "kernels.h"

using namespace dash;

struct dash_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    char* ws = nullptr;
    size_t ws_bytes = 0;
    char err[512] = {0};
    // statistics
    int64_t mm_products = 0, mm_launches = 0;
    double mm_block_products = 0.0;
    bool timing = false;
    std::vector<hipEvent_t> ev_pool;   // start/stop pairs
    std::vector<int> ev_variant;       // kernel variant of each pair
    size_t ev_used = 0;
    double ms_done = 0.0;
    int64_t var_launches[4] = {0, 0, 0, 0};
    double var_block_products[4] = {0, 0, 0, 0};
    double var_ms[4] = {0, 0, 0, 0};
    double mm_flops = 0.0;                       // flops of the tiles actually computed
    double var_flops[4] = {0, 0, 0, 0};
    // products that are symmetric in exact arithmetic compute only their upper triangle of tiles
    bool symmetric = true;
    int half_kind = HALF_BF16;      // 16-bit operand format of the call in progress (HALF_BF16 / HALF_FP16)
    // multi-Power-Iteration scaling: pool size, sweeps, start vectors [pi_rows][pi_pool] on the device
    int pi_pool = 0, pi_sweeps = 0, pi_rows = 0;
    const float* pi_v0 = nullptr;
    // this device's copy of the file-scope scratch array (its device address, resolved in dash_create)
    float* static_scratch = nullptr;
    // Lanes.  Launches on stacks of small blocks (B <= 512) are short -- one round of workgroups or less -- so
    // the fixed costs of a round (first operand loads, epilogue, ramp-up and tail) are a tenth and more of their
    // time.  Blocks are independent, so the iterative part of dash_inverse_root cuts such a chunk into two halves
    // ("lanes") that go through the same launch sequence on two streams: the context's and `aux`, a stream the
    // library owns (default priority), forked from and joined back into the context's stream with events, so
    // that one half's fixed costs fall into the other half's matrix-core time.  Results do not change by a bit.
    hipStream_t aux = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    int lanes = 1;                  // lanes of the chunk in progress (1: everything on the context's stream)
    bool use_lanes = true;          // dash_set_lanes
};

// Scratch of dash_block_norms_static: the slab partial sums of up to DASH_STATIC_MAX_BLOCKS blocks (32 per
// block), 2 MiB, held by every GPU the library runs on until the process ends.  In host code this name is
// only a handle for hipGetSymbolAddress; kernels and host calls use the address resolved per device.
constexpr int64_t STATIC_MAX_BLOCKS = 16384;
constexpr int STATIC_SLABS = 32;
static __device__ __align__(256) float scratch[STATIC_MAX_BLOCKS * STATIC_SLABS];

namespace {

typedef unsigned short bf16_t;   // host side only ever moves bf16 buffers around

constexpr size_t SCALARS_PER_BLOCK = 512;   // bytes of per-block scalars (slab partials, s, 1/s, s^(-1/p))
constexpr size_t WS_ALIGN = 256;

dash_status fail(dash_ctx* c, dash_status s, const char* fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof(c->err), fmt, ap);
        va_end(ap);
    }
    return s;
}

#define HIP_TRY(ctx, expr)                                                                   \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return fail(ctx, DASH_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));   \
    } while (0)

#define DASH_TRY(expr)                     \
    do {                                   \
        dash_status s_ = (expr);           \
        if (s_ != DASH_OK) return s_;      \
    } while (0)

bool valid_B(int B) { return B > 0 && B % 64 == 0 && B <= 16384; }

bool overlap(const void* a, const void* b, size_t bytes) {
    const char* x = (const char*)a;
    const char* y = (const char*)b;
    return x < y + bytes && y < x + bytes;
}

bool overlap2(const void* a, size_t abytes, const void* b, size_t bbytes) {
    const char* x = (const char*)a;
    const char* y = (const char*)b;
    return x < y + bbytes && y < x + abytes;
}

// per-block scratch of the scaling step: slab partials, s, 1/s, s^(-1/p), and the pool
// vectors / products / quotients of the multi-Power-Iteration
size_t scale_scratch_bytes(int B) {
    return SCALARS_PER_BLOCK + (power_iteration_bytes_per_block(B) + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN;
}

// fp32 and bf16 [B][B] buffers per block each method keeps in the workspace:
//   fp32 path: Newton-DB 5 fp32 (Y, Z ping-pong, E), Clenshaw 3 fp32 (S and two rotating B_k);
//   bf16 path: Newton-DB 5 bf16 (same roles) + 1 fp32 (the Y handed from call 1 to call 2),
//              Clenshaw 2 fp32 (rotating B_k) + 3 bf16 (S and the operand copies of B_k).
//   Coupled-Newton (fp32 only): 9 fp32 (X', M ping-pong, three C, C^2, C^4).
int f32_buffers(dash_method m, dash_precision prec) {
    if (m == DASH_COUPLED_NEWTON) return prec == DASH_FP32 ? 9 : 0;
    if (prec != DASH_FP32) return m == DASH_NEWTON_DB ? 1 : 2;
    return m == DASH_NEWTON_DB ? 5 : 3;
}
int bf16_buffers(dash_method m, dash_precision prec) {
    if (prec == DASH_FP32) return 0;
    // 16-bit iterates: five (Newton-DB), nine (Coupled-Newton), S and two B_k (Clenshaw); one, two or three planes each
    const int iterates = m == DASH_NEWTON_DB ? 5 : m == DASH_COUPLED_NEWTON ? 9 : 3;
    const int planes = prec == DASH_BF16X6 ? 3 : (prec == DASH_BF16X3 || prec == DASH_FP16X3) ? 2 : 1;
    return iterates * planes;
}

size_t per_block_bytes(int B, dash_method m, dash_precision prec) {
    size_t mat = (size_t)B * B * sizeof(float);
    return (size_t)f32_buffers(m, prec) * mat + (size_t)bf16_buffers(m, prec) * (mat / 2) + scale_scratch_bytes(B);
}

// ---- matmul launch with statistics / optional event timing ------------------------------
// blocks [off, off + cnt) of an n-block chunk that lane `lane` of `lanes` handles, and the stream it runs on
inline void lane_range(int64_t n, int lane, int lanes, int64_t* off, int64_t* cnt) {
    *off = n * lane / lanes;
    *cnt = n * (lane + 1) / lanes - *off;
}
inline hipStream_t lane_stream(const dash_ctx* c, int lane) { return lane == 0 ? c->stream : c->aux; }

dash_status run_gemm(dash_ctx* c, const GemmLaunch& g) {
    if (g.nblocks <= 0) return DASH_OK;
    const int variant = 2 * (g.prob[0].transA ? 1 : 0) + (g.prob[0].transB ? 1 : 0);
    const int lanes = g.nblocks >= 2 ? c->lanes : 1;
    double fl = 0.0;
    for (int lane = 0; lane < lanes; ++lane) {
        GemmLaunch gl = g;
        int64_t off, cnt;
        lane_range(g.nblocks, lane, lanes, &off, &cnt);
        gl.blk0 = g.blk0 + off;
        gl.nblocks = cnt;
        hipStream_t st = lane_stream(c, lane);
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (c->timing) {
            if (c->ev_used + 2 > c->ev_pool.size()) {
                for (int i = 0; i < 2; ++i) {
                    hipEvent_t e;
                    HIP_TRY(c, hipEventCreate(&e));
                    c->ev_pool.push_back(e);
                }
            }
            e0 = c->ev_pool[c->ev_used];
            e1 = c->ev_pool[c->ev_used + 1];
            if (c->ev_variant.size() < c->ev_pool.size() / 2) c->ev_variant.resize(c->ev_pool.size() / 2);
            c->ev_variant[c->ev_used / 2] = variant;
            c->ev_used += 2;
            HIP_TRY(c, hipEventRecord(e0, st));
        }
        HIP_TRY(c, launch_gemm(gl, st));
        if (c->timing) HIP_TRY(c, hipEventRecord(e1, st));
        fl += (double)gl.nprob * (double)gl.nblocks * 2.0 * (gl.M ? gl.M : gl.B) * (double)(gl.N ? gl.N : gl.B) *
              (gl.K ? gl.K : gl.B) * gemm_tile_fraction(gl);
    }
    // statistics count the launch once, whatever the number of lanes it was cut into
    c->mm_products += g.nprob;
    c->mm_launches += 1;
    c->mm_block_products += (double)g.nprob * (double)g.nblocks;
    c->var_launches[variant] += 1;
    c->var_block_products[variant] += (double)g.nprob * (double)g.nblocks;
    c->mm_flops += fl;
    c->var_flops[variant] += fl;
    return DASH_OK;
}

// launch_scale_shift on every lane of the chunk (same arguments; `stream` is replaced by the lane's)
hipError_t lane_scale_shift(dash_ctx* c, const float* in, int64_t n, int B, float eps, const float* mult, float a1, float g1,
                            float* out1, float a2, float g2, float* out2, void* h1, void* h2, int32_t* nonfinite,
                            hipStream_t /*stream*/, int half = HALF_BF16, void* l1 = nullptr, void* l2 = nullptr,
                            void* ll1 = nullptr, void* ll2 = nullptr) {
    const int lanes = n >= 2 ? c->lanes : 1;
    for (int lane = 0; lane < lanes; ++lane) {
        int64_t off, cnt;
        lane_range(n, lane, lanes, &off, &cnt);
        const size_t o = (size_t)off * B * B;
        auto f = [&](float* q) { return q ? q + o : nullptr; };
        auto h = [&](void* q) -> void* { return q ? static_cast<unsigned short*>(q) + o : nullptr; };
        hipError_t e = launch_scale_shift(in + o, cnt, B, eps, mult ? mult + off : nullptr, a1, g1, f(out1), a2, g2, f(out2),
                                          h(h1), h(h2), nonfinite ? nonfinite + off : nullptr, lane_stream(c, lane), half,
                                          h(l1), h(l2), h(ll1), h(ll2));
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

dash_status collect_events(dash_ctx* c) {
    if (c->ev_used == 0) return DASH_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, c->ev_pool[i], c->ev_pool[i + 1]));
        c->ms_done += ms;
        c->var_ms[c->ev_variant[i / 2]] += ms;
    }
    c->ev_used = 0;
    return DASH_OK;
}

GemmProblem problem(const float* A, const float* B, const float* D, float* C, const float* mult, float alpha,
                    float beta, float gamma, int ta = 0, int tb = 0) {
    GemmProblem p;
    p.A = A; p.B = B; p.D = D; p.C = C; p.Ch = nullptr; p.C2 = nullptr; p.C2h = nullptr; p.A2 = nullptr; p.B2 = nullptr; p.Cl = nullptr; p.A3 = nullptr; p.B3 = nullptr; p.Cl2 = nullptr; p.C2l = nullptr; p.C2l2 = nullptr; p.a2 = 0.f; p.g2 = 0.f; p.mult = mult;
    p.alpha = alpha; p.beta = beta; p.gamma = gamma; p.transA = ta; p.transB = tb;
    return p;
}

// bf16 operands Ah, Bh; result to C (fp32, may be null) and Ch (bf16, may be null)
GemmProblem problem_h(const bf16_t* Ah, const bf16_t* Bh, const float* D, float* C, bf16_t* Ch, const float* mult,
                      float alpha, float beta, float gamma, int ta = 0, int tb = 0) {
    GemmProblem p;
    p.A = Ah; p.B = Bh; p.D = D; p.C = C; p.Ch = Ch; p.C2 = nullptr; p.C2h = nullptr; p.A2 = nullptr; p.B2 = nullptr; p.Cl = nullptr; p.A3 = nullptr; p.B3 = nullptr; p.Cl2 = nullptr; p.C2l = nullptr; p.C2l2 = nullptr; p.a2 = 0.f; p.g2 = 0.f; p.mult = mult;
    p.alpha = alpha; p.beta = beta; p.gamma = gamma; p.transA = ta; p.transB = tb;
    return p;
}

// sym: the product is symmetric in exact arithmetic (see GemmLaunch::sym); honoured only while the
// context's symmetric mode is on
dash_status gemm1(dash_ctx* c, const GemmProblem& p, int64_t n, int B, int32_t* nonfinite = nullptr, int bf16 = 0,
                  bool sym = false) {
    GemmLaunch g;
    memset(&g, 0, sizeof(g));
    g.prob[0] = p; g.prob[1] = p; g.nprob = 1; g.B = B; g.nblocks = n; g.nonfinite = nonfinite; g.half = bf16 ? c->half_kind : HALF_NONE;
    g.sym = (sym && c->symmetric) ? 1 : 0;
    return run_gemm(c, g);
}

dash_status gemm2(dash_ctx* c, const GemmProblem& p0, const GemmProblem& p1, int64_t n, int B, int bf16 = 0,
                  bool sym = false) {
    GemmLaunch g;
    memset(&g, 0, sizeof(g));
    g.prob[0] = p0; g.prob[1] = p1; g.nprob = 2; g.B = B; g.nblocks = n; g.nonfinite = nullptr; g.half = bf16 ? c->half_kind : HALF_NONE;
    g.sym = (sym && c->symmetric) ? 1 : 0;
    return run_gemm(c, g);
}

// ---- workspace carving -----------------------------------------------------------------
struct Carve {
    char* p;
    char* end;
    void* take(size_t bytes) {
        size_t a = (bytes + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN;
        if (p + a > end) return nullptr;
        void* r = p;
        p += a;
        return r;
    }
};

// ---- scaling step (paper Sections 3.4, 3.5) on one chunk -----------------------------------
struct ScaleScratch {
    float *partial, *s, *inv_s, *unscale, *piV, *piW, *piq;
    bool carve(Carve& cv, int64_t nb, int B) {
        partial = (float*)cv.take((size_t)nb * norm_slabs(B) * sizeof(float));
        s = (float*)cv.take((size_t)nb * sizeof(float));
        inv_s = (float*)cv.take((size_t)nb * sizeof(float));
        unscale = (float*)cv.take((size_t)nb * sizeof(float));
        piV = (float*)cv.take((size_t)nb * B * 32 * sizeof(float));
        piW = (float*)cv.take((size_t)nb * B * 32 * sizeof(float));
        piq = (float*)cv.take((size_t)nb * power_iteration_q_floats(B) * sizeof(float));
        return partial && s && inv_s && unscale && piV && piW && piq;
    }
};

// s_b (to s_dst), 1/s_b and s_b^(-1/p) for the nb blocks at A
dash_status compute_scales(dash_ctx* c, const float* A, int64_t nb, int B, float eps, dash_scaling scaling, int p,
                           ScaleScratch& sc, float* s_dst) {
    hipStream_t st = c->stream;
    if (scaling == DASH_SCALE_POWER_ITERATION) {
        if (!c->pi_v0 || c->pi_pool < 1 || c->pi_sweeps < 1)
            return fail(c, DASH_ERR_INVALID_ARG, "power-iteration scaling needs dash_set_power_iteration first");
        if (c->pi_rows < B)
            return fail(c, DASH_ERR_INVALID_ARG, "start vectors have %d rows, blocks have %d", c->pi_rows, B);
        HIP_TRY(c, launch_power_iteration(A, nb, B, eps, c->pi_v0, c->pi_pool, c->pi_sweeps, p, sc.piV, sc.piW, sc.piq,
                                          s_dst, sc.inv_s, sc.unscale, st));
        return DASH_OK;
    }
    if (scaling != DASH_SCALE_NONE) HIP_TRY(c, launch_norm_partials(A, nb, B, eps, (int)scaling, sc.partial, st));
    HIP_TRY(c, launch_finalize_scale(sc.partial, nb, norm_slabs(B), (int)scaling, p, s_dst, sc.inv_s, sc.unscale, st));
    return DASH_OK;
}

// ---- Newton-DB on one chunk (paper Section 3.3) -----------------------------------------
// Symmetric mode touches only the residual product Z Y of E = 1.5 I - 0.5 Z Y.  The updates
// Y E and E Z are always computed in full: mirroring them (or symmetrising them in any way)
// breaks the coupling Y_k = A Z_k that keeps the iteration stable, and ill-conditioned
// blocks then diverge a few iterations after convergence.
// One call: from the input M (already scaled so that its spectrum lies in (0,1]) run
// `iters` updates of (Y, Z); the first is the closed form E_1 = 3/2 I - 1/2 M, Z_1 = E_1,
// Y_1 = M E_1.  keepY: the caller wants Y_k (first call of p = 4), otherwise Z_k.  The
// iterate that is not wanted is not computed in the last iteration (its value is unused),
// which saves one product per call relative to 3k-2.
// M is buf[mi]; on return *out_idx names the buffer with the wanted iterate, unless
// `final_out` is given: then the wanted Z_k is written there, multiplied by unscale_b.
dash_status ndb_call(dash_ctx* c, float* buf[5], int mi, int64_t n, int B, int iters, bool keepY,
                     bool m_needs_init, const float* A_in, float eps, const float* inv_s, float* final_out,
                     const float* unscale, int32_t* nonfinite, int* out_idx) {
    hipStream_t st = c->stream;
    // free list management over the 5 buffers
    bool used[5] = {false, false, false, false, false};
    auto grab = [&]() { for (int i = 0; i < 5; ++i) if (!used[i]) { used[i] = true; return i; } return -1; };
    int y, z;
    if (m_needs_init) {
        // first call: M = (A + eps I)/s -> buf[y]; E_1 = 1.5 I - 0.5 M -> buf[z]
        y = grab(); z = grab();
        HIP_TRY(c, lane_scale_shift(c, A_in, n, B, eps, inv_s, 1.f, 0.f, buf[y], -0.5f, 1.5f, buf[z], nullptr, nullptr, nullptr, st));
    } else {
        // chained call: M is buf[mi] as it stands; E_1 = 1.5 I - 0.5 M
        used[mi] = true; y = mi; z = grab();
        HIP_TRY(c, lane_scale_shift(c, buf[y], n, B, 0.f, nullptr, -0.5f, 1.5f, buf[z], 0.f, 0.f, nullptr, nullptr, nullptr, nullptr, st));
    }
    if (iters == 1) {
        if (keepY) {
            int y1 = grab();
            DASH_TRY(gemm1(c, problem(buf[y], buf[z], nullptr, buf[y1], nullptr, 1.f, 0.f, 0.f), n, B));
            *out_idx = y1;
        } else if (final_out) {
            // X = unscale * Z_1: no product at all
            HIP_TRY(c, lane_scale_shift(c, buf[z], n, B, 0.f, unscale, 1.f, 0.f, final_out, 0.f, 0.f, nullptr, nullptr, nullptr, nonfinite, st));
        } else {
            *out_idx = z;
        }
        return DASH_OK;
    }
    {   // Y_1 = M E_1
        int y1 = grab();
        DASH_TRY(gemm1(c, problem(buf[y], buf[z], nullptr, buf[y1], nullptr, 1.f, 0.f, 0.f), n, B));
        used[y] = false; y = y1;
    }
    for (int it = 2; it <= iters; ++it) {
        const bool last = it == iters;
        int e = grab();
        // E = 1.5 I - 0.5 Z Y
        DASH_TRY(gemm1(c, problem(buf[z], buf[y], nullptr, buf[e], nullptr, -0.5f, 0.f, 1.5f), n, B, nullptr, 0, true));
        if (!last) {
            int y2 = grab(), z2 = grab();
            DASH_TRY(gemm2(c, problem(buf[y], buf[e], nullptr, buf[y2], nullptr, 1.f, 0.f, 0.f),
                           problem(buf[e], buf[z], nullptr, buf[z2], nullptr, 1.f, 0.f, 0.f), n, B));
            used[y] = used[z] = used[e] = false;
            y = y2; z = z2;
        } else if (keepY) {
            int y2 = grab();
            DASH_TRY(gemm1(c, problem(buf[y], buf[e], nullptr, buf[y2], nullptr, 1.f, 0.f, 0.f), n, B));
            *out_idx = y2;
        } else if (final_out) {
            DASH_TRY(gemm1(c, problem(buf[e], buf[z], nullptr, final_out, unscale, 1.f, 0.f, 0.f), n, B, nonfinite));
        } else {
            int z2 = grab();
            DASH_TRY(gemm1(c, problem(buf[e], buf[z], nullptr, buf[z2], nullptr, 1.f, 0.f, 0.f), n, B));
            *out_idx = z2;
        }
    }
    return DASH_OK;
}

// ---- Newton-DB with bf16 operands (Appendix A.3 recipe applied to Section 3.3) ------------
// Every iterate is consumed only as a matmul operand, i.e. only after rounding to bf16, so
// the iterates live in the workspace as the bf16 values the next product reads; the fp32
// value is kept where something else reads it: the Y that call 1 hands to call 2 (its
// closed-form E_1 is formed from the fp32 Y) and the final Z (the result).  Accumulation
// and every epilogue (1.5 I - 0.5 Z Y, un-scaling) are fp32.
// hb: five bf16 buffers; fy: one fp32 buffer.  mi: index in hb of the bf16 copy of M when
// the call is chained (then fy holds M in fp32).
dash_status ndb_call_bf16(dash_ctx* c, bf16_t* hb[5], bf16_t** lb, bf16_t** lb2, float* fy, int mi, int64_t n, int B, int iters,
                          bool keepY, bool m_needs_init, const float* A_in, float eps, const float* inv_s,
                          float* final_out, const float* unscale, int32_t* nonfinite, int* out_idx) {
    // lb != null: split-operand mode, every iterate is kept as a high plane hb[i] and a low plane lb[i]
    // (x ~ hi + lo), products are A_lo B_hi + A_hi B_lo + A_hi B_hi; lb2 != null as well: three planes
    // (x ~ hi + mid + lo, lb the middle and lb2 the lowest plane) and six-term products
    hipStream_t st = c->stream;
    bool used[5] = {false, false, false, false, false};
    auto grab = [&]() { for (int i = 0; i < 5; ++i) if (!used[i]) { used[i] = true; return i; } return -1; };
    auto lo = [&](int i) -> bf16_t* { return lb ? lb[i] : nullptr; };
    auto lo2 = [&](int i) -> bf16_t* { return lb2 ? lb2[i] : nullptr; };
    // product of iterates ia, ib -> iterate ic (16-bit planes) and/or Cf (fp32)
    auto prod = [&](int ia, int ib, float* Cf, int ic, const float* mult, float alpha, float gamma) {
        GemmProblem p = problem_h(hb[ia], hb[ib], nullptr, Cf, ic >= 0 ? hb[ic] : nullptr, mult, alpha, 0.f, gamma);
        p.A2 = lo(ia); p.B2 = lo(ib); p.Cl = ic >= 0 ? lo(ic) : nullptr;
        p.A3 = lo2(ia); p.B3 = lo2(ib); p.Cl2 = ic >= 0 ? lo2(ic) : nullptr;
        return p;
    };
    int y, z;
    if (m_needs_init) {
        y = grab(); z = grab();
        // M = (A + eps I)/s -> planes of y; E_1 = 1.5 I - 0.5 M (fp32) -> planes of z; when E_1 itself is
        // the result (iters == 1, p == 2) its fp32 value goes to fy
        HIP_TRY(c, lane_scale_shift(c, A_in, n, B, eps, inv_s, 1.f, 0.f, nullptr, -0.5f, 1.5f,
                                      (iters == 1 && !keepY) ? fy : nullptr, hb[y], hb[z], nullptr, st, c->half_kind,
                                      lo(y), lo(z), lo2(y), lo2(z)));
    } else {
        used[mi] = true; y = mi; z = grab();
        if (iters == 1 && !keepY && final_out) {
            // X = unscale * (1.5 I - 0.5 Y): two elementwise passes, no product
            HIP_TRY(c, lane_scale_shift(c, fy, n, B, 0.f, nullptr, -0.5f, 1.5f, final_out, 0.f, 0.f, nullptr, nullptr,
                                          nullptr, nullptr, st, c->half_kind));
            HIP_TRY(c, lane_scale_shift(c, final_out, n, B, 0.f, unscale, 1.f, 0.f, final_out, 0.f, 0.f, nullptr,
                                          nullptr, nullptr, nonfinite, st, c->half_kind));
            return DASH_OK;
        }
        HIP_TRY(c, lane_scale_shift(c, fy, n, B, 0.f, nullptr, -0.5f, 1.5f, nullptr, 0.f, 0.f, nullptr, hb[z], nullptr,
                                      nullptr, st, c->half_kind, lo(z), nullptr, lo2(z), nullptr));
    }
    if (iters == 1) {
        if (keepY) {
            int y1 = grab();
            DASH_TRY(gemm1(c, prod(y, z, fy, y1, nullptr, 1.f, 0.f), n, B, nullptr, 1));
            *out_idx = y1;
        } else if (final_out) {
            HIP_TRY(c, lane_scale_shift(c, fy, n, B, 0.f, unscale, 1.f, 0.f, final_out, 0.f, 0.f, nullptr, nullptr,
                                          nullptr, nonfinite, st, c->half_kind));
        } else {
            *out_idx = z;
        }
        return DASH_OK;
    }
    {
        int y1 = grab();
        DASH_TRY(gemm1(c, prod(y, z, nullptr, y1, nullptr, 1.f, 0.f), n, B, nullptr, 1));
        used[y] = false; y = y1;
    }
    for (int it = 2; it <= iters; ++it) {
        const bool last = it == iters;
        int e = grab();
        DASH_TRY(gemm1(c, prod(z, y, nullptr, e, nullptr, -0.5f, 1.5f), n, B, nullptr, 1, true));
        if (!last) {
            int y2 = grab(), z2 = grab();
            DASH_TRY(gemm2(c, prod(y, e, nullptr, y2, nullptr, 1.f, 0.f), prod(e, z, nullptr, z2, nullptr, 1.f, 0.f), n, B, 1));
            used[y] = used[z] = used[e] = false;
            y = y2; z = z2;
        } else if (keepY) {
            int y2 = grab();
            DASH_TRY(gemm1(c, prod(y, e, fy, y2, nullptr, 1.f, 0.f), n, B, nullptr, 1));
            *out_idx = y2;
        } else if (final_out) {
            DASH_TRY(gemm1(c, prod(e, z, final_out, -1, unscale, 1.f, 0.f), n, B, nonfinite, 1));
        } else {
            int z2 = grab();
            DASH_TRY(gemm1(c, prod(e, z, nullptr, z2, nullptr, 1.f, 0.f), n, B, nullptr, 1));
            *out_idx = z2;
        }
    }
    return DASH_OK;
}

// ---- Clenshaw with bf16 operands (paper Appendix A.3: B_k kept in fp32, S and the operand
// copy of B_{k+1} in half precision, fp32 accumulation) ----------------------------------------
dash_status clenshaw_chunk_bf16(dash_ctx* c, float* fb[2], bf16_t* hb[3], const float* A, float* X, int64_t n, int B,
                                int d, const double* cf, double ca, double cb, float eps, const float* inv_s,
                                const float* unscale, int32_t* nonfinite, bf16_t** hm = nullptr, bf16_t** hl = nullptr) {
    // hm, hl != null: three-plane mode -- the operand copies of S, B_{k+1}, B_{k+2} are carried as three bf16
    // planes each (hb the high, hm the middle, hl the lowest planes) and every product has six segments
    hipStream_t st = c->stream;
    int i1 = 1, i2 = 2;                       // plane sets of B_{k+1} and B_{k+2} (set 0 is S)
    float* b1 = fb[0];                        // B_{k+1}: fp32 master next to its operand copy
    float* b2 = fb[1];                        // B_{k+2}
    auto mid = [&](int i) -> bf16_t* { return hm ? hm[i] : nullptr; };
    auto low = [&](int i) -> bf16_t* { return hl ? hl[i] : nullptr; };
    // S B_{k+1} (operand copies) with D, fp32 result Cf and operand copy of the result in plane set ic (-1: none)
    auto prod = [&](const float* D, float* Cf, int ic, const float* mult, float alpha, float beta, float gamma) {
        GemmProblem p = problem_h(hb[0], hb[i1], D, Cf, ic >= 0 ? hb[ic] : nullptr, mult, alpha, beta, gamma);
        p.A2 = mid(0); p.B2 = mid(i1); p.Cl = ic >= 0 ? mid(ic) : nullptr;
        p.A3 = low(0); p.B3 = low(i1); p.Cl2 = ic >= 0 ? low(ic) : nullptr;
        return p;
    };
    const float m1 = (float)(2.0 / (cb - ca)), m0 = (float)(-(ca + cb) / (cb - ca));
    HIP_TRY(c, lane_scale_shift(c, A, n, B, eps, inv_s, m1, m0, nullptr, (float)(2.0 * cf[d]), (float)cf[d - 1], b1,
                                  hb[0], hb[i1], nullptr, st, c->half_kind, mid(0), mid(i1), low(0), low(i1)));
    if (d == 2)
        return gemm1(c, prod(nullptr, X, -1, unscale, 1.f, 0.f, (float)(cf[0] - cf[2])), n, B, nonfinite, 1, true);
    DASH_TRY(gemm1(c, prod(nullptr, b2, i2, nullptr, 2.f, 0.f, (float)(cf[d - 2] - cf[d])), n, B, nullptr, 1, true));
    { float* t = b1; b1 = b2; b2 = t; int u = i1; i1 = i2; i2 = u; }
    for (int k = d - 3; k >= 1; --k) {
        DASH_TRY(gemm1(c, prod(b2, b2, i2, nullptr, 2.f, -1.f, (float)cf[k]), n, B, nullptr, 1, true));
        float* t = b1; b1 = b2; b2 = t; int u = i1; i1 = i2; i2 = u;
    }
    return gemm1(c, prod(b2, X, -1, unscale, 1.f, -1.f, (float)cf[0]), n, B, nonfinite, 1, true);
}

// ---- Coupled-Newton on one chunk (paper Section 3.2) ----------------------------------------
//   X_0 = I/c, M_0 = A_s/c^p, C_k = (1+1/p) I - M_k/p, X_{k+1} = X_k C_k, M_{k+1} = C_k^p M_k,
//   c = (1+p)^(-1/p) so that M_0 = (p+1) A_s.
// The constant 1/c is carried in the final multiplier (X_k = (1/c) C_0 ... C_{k-1}), so the first
// update X_1 needs no product; the last iteration computes only X (nobody reads its M), so k
// iterations cost (k-1) * (3 or 4) products against the paper's k * (3 or 4).  C_{k+1} is written by
// the epilogue of the M product.  Every product is computed in full whatever the symmetric mode says:
// mirroring even only the powers C^2, C^4 makes X drift after convergence (measured at kappa = 1e4:
// 3.7e-3 after 40 iterations, 9e-3 after 80, against a steady 9.4e-5 with full products).
// buf: 9 fp32 buffers (X' x2, M x2, C x3, C^2, C^4).  s_b^(-1/p) / c is applied in the last epilogue.  C_k lives in Cb[k % 3]: the launch that reads C_k (and, for k = 1, C_0 in its role as X'_1)
// writes C_{k+1} into the third buffer.
dash_status cn_chunk(dash_ctx* c, float* buf[9], const float* A, float* X, int64_t n, int B, int p, int iters,
                     float eps, const float* inv_s, const float* unscale, int32_t* nonfinite) {
    hipStream_t st = c->stream;
    const float a = 1.f + 1.f / p, ip = 1.f / p;
    const float inv_c = (float)std::pow(1.0 + p, 1.0 / p);      // 1/c with c = (1+p)^(-1/p)
    float* Xb[2] = {buf[0], buf[1]};
    float* Mb[2] = {buf[2], buf[3]};
    float* Cb[3] = {buf[4], buf[5], buf[6]};
    float *P2 = buf[7], *P4 = buf[8];
    // M_0 = (p+1) (A + eps I)/s ; C_0 = a I - M_0/p
    HIP_TRY(c, lane_scale_shift(c, A, n, B, eps, inv_s, (float)(p + 1), 0.f, Mb[0], -ip, a, Cb[0], nullptr, nullptr,
                                  nullptr, st));
    if (iters == 1) {   // X = s^(-1/p) (1/c) C_0, no product
        HIP_TRY(c, lane_scale_shift(c, Cb[0], n, B, 0.f, unscale, inv_c, 0.f, X, 0.f, 0.f, nullptr, nullptr, nullptr,
                                      nonfinite, st));
        return DASH_OK;
    }
    const float* Xcur = Cb[0];          // X'_1 = C_0
    for (int k = 0; k + 1 < iters; ++k) {
        float* Ck = Cb[k % 3];
        // C_k^p by repeated squaring
        DASH_TRY(gemm1(c, problem(Ck, Ck, nullptr, P2, nullptr, 1.f, 0.f, 0.f), n, B));
        const float* Pp = P2;
        if (p == 4) {
            DASH_TRY(gemm1(c, problem(P2, P2, nullptr, P4, nullptr, 1.f, 0.f, 0.f), n, B));
            Pp = P4;
        }
        // M_{k+1} = C_k^p M_k with C_{k+1} = a I - M_{k+1}/p from the same epilogue
        GemmProblem pm = problem(Pp, Mb[k % 2], nullptr, Mb[(k + 1) % 2], nullptr, 1.f, 0.f, 0.f);
        pm.C2 = Cb[(k + 1) % 3]; pm.a2 = -ip; pm.g2 = a;
        if (k == 0) {
            DASH_TRY(gemm1(c, pm, n, B));                       // X'_1 = C_0 needs no product
        } else {
            float* Xn = Xb[k % 2];                              // X'_{k+1} = X'_k C_k in the same launch
            DASH_TRY(gemm2(c, pm, problem(Xcur, Ck, nullptr, Xn, nullptr, 1.f, 0.f, 0.f), n, B));
            Xcur = Xn;
        }
    }
    // last update, un-scaled: X = s^(-1/p) (1/c) X'_{iters-1} C_{iters-1}
    return gemm1(c, problem(Xcur, Cb[(iters - 1) % 3], nullptr, X, unscale, inv_c, 0.f, 0.f), n, B, nonfinite);
}

// Coupled-Newton with 16-bit operands (the paper's fastest configuration is Coupled-Newton in fp16,
// Sections 2.3 and 5): every iterate is read only as a matmul operand (C_{k+1} is formed from the fp32
// accumulator of the M product before rounding), so all nine buffers hold 16-bit values; accumulation,
// the epilogue arithmetic and the result X are fp32.
dash_status cn_chunk_half(dash_ctx* c, bf16_t* hb[9], const float* A, float* X, int64_t n, int B, int p, int iters,
                          float eps, const float* inv_s, const float* unscale, int32_t* nonfinite, float* tmp_f32,
                          bf16_t** hm = nullptr, bf16_t** hl = nullptr) {
    // hm, hl != null: three-plane mode -- every iterate is carried as three bf16 planes (hb the high, hm the
    // middle, hl the lowest planes of the same nine iterates) and every product has six segments
    hipStream_t st = c->stream;
    const float a = 1.f + 1.f / p, ip = 1.f / p;
    const float inv_c = (float)std::pow(1.0 + p, 1.0 / p);
    // iterate indices: X ping-pong 0, 1; M ping-pong 2, 3; three C 4, 5, 6; C^2 7; C^4 8
    auto mid = [&](int i) -> bf16_t* { return hm && i >= 0 ? hm[i] : nullptr; };
    auto low = [&](int i) -> bf16_t* { return hl && i >= 0 ? hl[i] : nullptr; };
    // iterate ia times iterate ib -> iterate ic (-1: none) and/or fp32 Cf
    auto prod = [&](int ia, int ib, float* Cf, int ic, const float* mult, float alpha) {
        GemmProblem q = problem_h(hb[ia], hb[ib], nullptr, Cf, ic >= 0 ? hb[ic] : nullptr, mult, alpha, 0.f, 0.f);
        q.A2 = mid(ia); q.B2 = mid(ib); q.Cl = mid(ic);
        q.A3 = low(ia); q.B3 = low(ib); q.Cl2 = low(ic);
        return q;
    };
    if (iters == 1) {   // X = s^(-1/p) (1/c) C_0 in fp32, no product: C_0 via the fp32 temporary X itself
        HIP_TRY(c, lane_scale_shift(c, A, n, B, eps, inv_s, (float)(p + 1), 0.f, nullptr, -ip, a, X, nullptr, nullptr,
                                      nullptr, st, c->half_kind));
        HIP_TRY(c, lane_scale_shift(c, X, n, B, 0.f, unscale, inv_c, 0.f, X, 0.f, 0.f, nullptr, nullptr, nullptr,
                                      nonfinite, st, c->half_kind));
        (void)tmp_f32;
        return DASH_OK;
    }
    HIP_TRY(c, lane_scale_shift(c, A, n, B, eps, inv_s, (float)(p + 1), 0.f, nullptr, -ip, a, nullptr, hb[2], hb[4],
                                  nullptr, st, c->half_kind, mid(2), mid(4), low(2), low(4)));
    int xcur = 4;                                   // X_1 = (1/c) C_0: the first update needs no product
    for (int k = 0; k + 1 < iters; ++k) {
        const int ck = 4 + k % 3;
        DASH_TRY(gemm1(c, prod(ck, ck, nullptr, 7, nullptr, 1.f), n, B, nullptr, 1));
        int pp = 7;
        if (p == 4) {
            DASH_TRY(gemm1(c, prod(7, 7, nullptr, 8, nullptr, 1.f), n, B, nullptr, 1));
            pp = 8;
        }
        const int cn = 4 + (k + 1) % 3;
        GemmProblem pm = prod(pp, 2 + k % 2, nullptr, 2 + (k + 1) % 2, nullptr, 1.f);
        pm.C2h = hb[cn]; pm.C2l = mid(cn); pm.C2l2 = low(cn); pm.a2 = -ip; pm.g2 = a;
        if (k == 0) {
            DASH_TRY(gemm1(c, pm, n, B, nullptr, 1));
        } else {
            const int xn = k % 2;
            DASH_TRY(gemm2(c, pm, prod(xcur, ck, nullptr, xn, nullptr, 1.f), n, B, 1));
            xcur = xn;
        }
    }
    return gemm1(c, prod(xcur, 4 + (iters - 1) % 3, X, -1, unscale, inv_c), n, B, nonfinite, 1);
}

// ---- Clenshaw on one chunk (paper Appendix A.2, reduced form, d-1 products) --------------
dash_status clenshaw_chunk(dash_ctx* c, float* buf[3], const float* A, float* X, int64_t n, int B, int d,
                           const double* cf, double ca, double cb, float eps, const float* inv_s,
                           const float* unscale, int32_t* nonfinite) {
    hipStream_t st = c->stream;
    float* S = buf[0];
    float* b1 = buf[1];   // B_{k+1}
    float* b2 = buf[2];   // B_{k+2}
    const float m1 = (float)(2.0 / (cb - ca)), m0 = (float)(-(ca + cb) / (cb - ca));
    // S = (2 A_s - (a+b) I)/(b-a);  B_{d-1} = 2 c_d S + c_{d-1} I.  B_d = c_d I is never stored:
    // it only enters B_{d-2} through "- B_d + c_{d-2} I" = (c_{d-2} - c_d) I.
    HIP_TRY(c, lane_scale_shift(c, A, n, B, eps, inv_s, m1, m0, S, (float)(2.0 * cf[d]), (float)cf[d - 1], b1,
                                  nullptr, nullptr, nullptr, st));
    if (d == 2) {
        // result = S B_1 - B_2 + c_0 I with B_2 = c_2 I
        return gemm1(c, problem(S, b1, nullptr, X, unscale, 1.f, 0.f, (float)(cf[0] - cf[2])), n, B, nonfinite, 0, true);
    }
    // k = d-2: B_{d-2} = 2 S B_{d-1} + (c_{d-2} - c_d) I
    DASH_TRY(gemm1(c, problem(S, b1, nullptr, b2, nullptr, 2.f, 0.f, (float)(cf[d - 2] - cf[d])), n, B, nullptr, 0, true));
    { float* t = b1; b1 = b2; b2 = t; }   // b1 = B_{d-2}, b2 = B_{d-1}
    for (int k = d - 3; k >= 1; --k) {
        // B_k = 2 S B_{k+1} - B_{k+2} + c_k I, written over B_{k+2}
        DASH_TRY(gemm1(c, problem(S, b1, b2, b2, nullptr, 2.f, -1.f, (float)cf[k]), n, B, nullptr, 0, true));
        float* t = b1; b1 = b2; b2 = t;
    }
    // result = S B_1 - B_2 + c_0 I, un-scaled
    return gemm1(c, problem(S, b1, b2, X, unscale, 1.f, -1.f, (float)cf[0]), n, B, nonfinite, 0, true);
}

// Two lanes for blocks of at most LANE_MAX_B when a single-product launch over the whole chunk would have at least
// LANE_MIN_TILES_* output tiles of 128 x 128 (fp32: one full round of resident workgroups; 16-bit launches are shorter
// and gain from a quarter of that).  Measured, lanes on against off: 256 blocks of 256 Newton-DB 3.70 -> 3.62 ms,
// Clenshaw 1.03 -> 0.89, two fp16 planes on 64 blocks of 256 0.93 -> 0.73; below the thresholds they lose (64 blocks of
// 128: 0.31 -> 0.36 ms), above B = 512 nothing is left to gain.
constexpr int LANE_MAX_B = 512;
constexpr int64_t LANE_MIN_TILES_FP32 = 1024, LANE_MIN_TILES_16BIT = 256;
inline bool chunk_takes_lanes(const dash_ctx* c, int64_t nb, int B, dash_precision precision) {
    if (!c->use_lanes || B > LANE_MAX_B || nb < 2) return false;
    const int64_t tiles = nb * B * B / (128 * 128);
    return tiles >= (precision == DASH_FP32 ? LANE_MIN_TILES_FP32 : LANE_MIN_TILES_16BIT);
}

// fork: the second lane's stream waits for everything enqueued so far on the context's stream; join: the context's
// stream waits for the second lane.  Both are event record / wait pairs (legal under stream capture: the second
// stream joins the capture at the fork and leaves it at the join).
struct LaneScope {
    dash_ctx* c;
    int lanes;
    bool forked = false;
    LaneScope(dash_ctx* ctx, int n) : c(ctx), lanes(n) {}
    dash_status fork() {
        if (lanes < 2) return DASH_OK;
        HIP_TRY(c, hipEventRecord(c->ev_fork, c->stream));
        HIP_TRY(c, hipStreamWaitEvent(c->aux, c->ev_fork, 0));
        forked = true;
        c->lanes = lanes;
        return DASH_OK;
    }
    dash_status join() {
        c->lanes = 1;
        if (!forked) return DASH_OK;
        forked = false;
        HIP_TRY(c, hipEventRecord(c->ev_join, c->aux));
        HIP_TRY(c, hipStreamWaitEvent(c->stream, c->ev_join, 0));
        return DASH_OK;
    }
    ~LaneScope() { if (forked) (void)join(); }
};

}  // namespace

// =========================================================================================
// public ABI
// =========================================================================================

extern "C" {

const char* dash_status_string(dash_status s) {
    switch (s) {
        case DASH_OK: return "ok";
        case DASH_ERR_INVALID_ARG: return "invalid argument";
        case DASH_ERR_UNSUPPORTED: return "unsupported";
        case DASH_ERR_WORKSPACE: return "workspace missing or too small";
        case DASH_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

dash_status dash_create(dash_ctx** out, int device, void* hip_stream) {
    if (!out) return DASH_ERR_INVALID_ARG;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return DASH_ERR_HIP;
    if (hipSetDevice(device) != hipSuccess) return DASH_ERR_HIP;
    dash_ctx* c = new (std::nothrow) dash_ctx();
    if (!c) return DASH_ERR_HIP;
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    // device address of this GPU's copy of the static scratch array (the device is current here)
    void* sp = nullptr;
    if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || !sp) {
        delete c;
        return DASH_ERR_HIP;
    }
    c->static_scratch = static_cast<float*>(sp);
    // the second lane's stream (default priority) and the events that fork it from and join it into the context's stream
    if (hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) {
        dash_destroy(c);
        return DASH_ERR_HIP;
    }
    *out = c;
    return DASH_OK;
}

dash_status dash_set_stream(dash_ctx* c, void* hip_stream) {
    if (!c) return DASH_ERR_INVALID_ARG;
    c->stream = (hipStream_t)hip_stream;
    return DASH_OK;
}

dash_status dash_destroy(dash_ctx* c) {
    if (!c) return DASH_ERR_INVALID_ARG;
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    if (c->aux) (void)hipStreamDestroy(c->aux);
    delete c;
    return DASH_OK;
}

size_t dash_workspace_bytes(int64_t n_blocks, int B, dash_method method, int p, dash_precision precision) {
    (void)p;
    if (n_blocks <= 0 || !valid_B(B)) return 0;
    return (size_t)n_blocks * per_block_bytes(B, method, precision) + 4 * WS_ALIGN * 16;
}

dash_status dash_set_workspace(dash_ctx* c, void* dev_ptr, size_t bytes) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (dev_ptr && ((uintptr_t)dev_ptr % WS_ALIGN)) return fail(c, DASH_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    c->ws = (char*)dev_ptr;
    c->ws_bytes = dev_ptr ? bytes : 0;
    return DASH_OK;
}

const char* dash_last_error(const dash_ctx* c) { return c ? c->err : "null context"; }

dash_status dash_reset_stats(dash_ctx* c) {
    if (!c) return DASH_ERR_INVALID_ARG;
    DASH_TRY(collect_events(c));
    c->mm_products = c->mm_launches = 0;
    c->mm_block_products = 0.0;
    c->ms_done = 0.0;
    for (int v = 0; v < 4; ++v) { c->var_launches[v] = 0; c->var_block_products[v] = 0.0; c->var_ms[v] = 0.0; c->var_flops[v] = 0.0; }
    c->mm_flops = 0.0;
    return DASH_OK;
}

dash_status dash_set_timing(dash_ctx* c, int on) {
    if (!c) return DASH_ERR_INVALID_ARG;
    DASH_TRY(collect_events(c));
    c->timing = on != 0;
    return DASH_OK;
}

dash_status dash_set_symmetric(dash_ctx* c, int on) {
    if (!c) return DASH_ERR_INVALID_ARG;
    c->symmetric = on != 0;
    return DASH_OK;
}

dash_status dash_set_lanes(dash_ctx* c, int on) {
    if (!c) return DASH_ERR_INVALID_ARG;
    c->use_lanes = on != 0;
    return DASH_OK;
}

dash_status dash_set_power_iteration(dash_ctx* c, int pool, int sweeps, const float* start_vectors, int rows) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (pool < 1 || pool > 32) return fail(c, DASH_ERR_INVALID_ARG, "pool must be in 1..32 (got %d)", pool);
    if (sweeps < 1) return fail(c, DASH_ERR_INVALID_ARG, "sweeps must be >= 1");
    if (!start_vectors || rows < 1) return fail(c, DASH_ERR_INVALID_ARG, "start vectors missing");
    c->pi_pool = pool; c->pi_sweeps = sweeps; c->pi_v0 = start_vectors; c->pi_rows = rows;
    return DASH_OK;
}

dash_status dash_get_stats(dash_ctx* c, dash_stats* out) {
    if (!c || !out) return DASH_ERR_INVALID_ARG;
    DASH_TRY(collect_events(c));
    out->matmul_products = c->mm_products;
    out->matmul_launches = c->mm_launches;
    out->matmul_block_products = c->mm_block_products;
    out->matmul_ms = c->ms_done;
    for (int v = 0; v < 4; ++v) {
        out->variant_launches[v] = c->var_launches[v];
        out->variant_block_products[v] = c->var_block_products[v];
        out->variant_ms[v] = c->var_ms[v];
        out->variant_flops[v] = c->var_flops[v];
    }
    out->matmul_flops = c->mm_flops;
    return DASH_OK;
}

dash_status dash_gemm_batched(dash_ctx* c, int transA, int transB, const float* A, const float* Bm, const float* D,
                              float* C, int64_t N, int B, float alpha, float beta, float gamma,
                              dash_precision precision) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64 (N=%lld B=%d)", (long long)N, B);
    if (N == 0) return DASH_OK;
    if (!A || !Bm || !C) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    if (!D && beta != 0.f) return fail(c, DASH_ERR_INVALID_ARG, "beta != 0 needs D");
    if (precision != DASH_FP32 && precision != DASH_BF16_ACC32 && precision != DASH_FP16_ACC32 && precision != DASH_BF16X3 &&
        precision != DASH_BF16X6 && precision != DASH_FP16X3)
        return fail(c, DASH_ERR_INVALID_ARG, "bad precision");
    c->half_kind = (precision == DASH_FP16_ACC32 || precision == DASH_FP16X3) ? HALF_FP16 : HALF_BF16;
    const bool planes3 = precision == DASH_BF16X6;
    const bool split = precision == DASH_BF16X3 || precision == DASH_FP16X3 || planes3;
    const size_t bytes = (size_t)N * B * B * sizeof(float);
    if (overlap(C, A, bytes) || overlap(C, Bm, bytes)) return fail(c, DASH_ERR_INVALID_ARG, "C overlaps an operand");
    if (D && D != C && overlap(C, D, bytes)) return fail(c, DASH_ERR_INVALID_ARG, "D must equal C or be disjoint from it");
    HIP_TRY(c, hipSetDevice(c->device));
    if (precision == DASH_FP32)
        return gemm1(c, problem(A, Bm, D, C, nullptr, alpha, beta, gamma, transA ? 1 : 0, transB ? 1 : 0), N, B);
    // 16-bit operands: round both operand stacks into the workspace (two 16-bit stacks per chunk, four or six in
    // the split modes: two or three planes each), then multiply
    const size_t mat = (size_t)B * B, per = (planes3 ? 6 : split ? 4 : 2) * mat * sizeof(bf16_t);
    if (!c->ws || c->ws_bytes < per) return fail(c, DASH_ERR_WORKSPACE, "workspace holds %zu bytes, one block needs %zu", c->ws_bytes, per);
    int64_t chunk = (int64_t)(c->ws_bytes / per);
    if (chunk > N) chunk = N;
    for (int64_t b0 = 0; b0 < N; b0 += chunk) {
        const int64_t nb = N - b0 < chunk ? N - b0 : chunk;
        const size_t o = (size_t)b0 * mat;
        bf16_t* Ah = (bf16_t*)c->ws;
        bf16_t* Bh = Ah + (size_t)nb * mat;
        bf16_t* Al = split ? Bh + (size_t)nb * mat : nullptr;
        bf16_t* Bl = split ? Al + (size_t)nb * mat : nullptr;
        bf16_t* Al2 = planes3 ? Bl + (size_t)nb * mat : nullptr;
        bf16_t* Bl2 = planes3 ? Al2 + (size_t)nb * mat : nullptr;
        HIP_TRY(c, launch_scale_shift(A + o, nb, B, 0.f, nullptr, 1.f, 0.f, nullptr, 0.f, 0.f, nullptr, Ah, nullptr, nullptr, c->stream, c->half_kind, Al, nullptr, Al2, nullptr));
        HIP_TRY(c, launch_scale_shift(Bm + o, nb, B, 0.f, nullptr, 1.f, 0.f, nullptr, 0.f, 0.f, nullptr, Bh, nullptr, nullptr, c->stream, c->half_kind, Bl, nullptr, Bl2, nullptr));
        GemmProblem pr = problem_h(Ah, Bh, D ? D + o : nullptr, C + o, nullptr, nullptr, alpha, beta, gamma,
                                   transA ? 1 : 0, transB ? 1 : 0);
        pr.A2 = Al; pr.B2 = Bl;
        pr.A3 = Al2; pr.B3 = Bl2;
        DASH_TRY(gemm1(c, pr, nb, B, nullptr, 1));
    }
    return DASH_OK;
}

dash_status dash_accumulate_factors(dash_ctx* c, const float* G, float* L, float* R, int64_t N, int B, float beta,
                                    float alpha) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64 (N=%lld B=%d)", (long long)N, B);
    if (N == 0) return DASH_OK;
    if (!G || !L || !R) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    const size_t bytes = (size_t)N * B * B * sizeof(float);
    if (overlap(L, G, bytes) || overlap(R, G, bytes) || overlap(L, R, bytes))
        return fail(c, DASH_ERR_INVALID_ARG, "G, L, R must not overlap");
    HIP_TRY(c, hipSetDevice(c->device));
    // L = beta L + alpha G G^T ; R = beta R + alpha G^T G  (EMA fused in the epilogue)
    // G G^T and G^T G are symmetric bit for bit (same products, same summation order for (i,j) and (j,i))
    // (one launch for both: the two products of a block use different memory orders of G)
    DASH_TRY(gemm2(c, problem(G, G, L, L, nullptr, alpha, beta, 0.f, 0, 1), problem(G, G, R, R, nullptr, alpha, beta, 0.f, 1, 0),
                   N, B, 0, true));
    return DASH_OK;
}

// ---- ragged gradient blocks (Section 4.1: G_rest of shape (N, Bm, Bn), L_rest (N, Bm, Bm), R_rest (N, Bn, Bn)) ----
dash_status dash_accumulate_factors_rect(dash_ctx* c, const float* G, float* L, float* R, int64_t N, int Bm, int Bn,
                                         float beta, float alpha) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(Bm) || !valid_B(Bn))
        return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and Bm, Bn multiples of 64 (N=%lld Bm=%d Bn=%d)", (long long)N, Bm, Bn);
    if (N == 0) return DASH_OK;
    if (!G || !L || !R) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    const size_t gb = (size_t)N * Bm * Bn * 4, lb = (size_t)N * Bm * Bm * 4, rb = (size_t)N * Bn * Bn * 4;
    if (overlap2(L, lb, G, gb) || overlap2(R, rb, G, gb) || overlap2(L, lb, R, rb))
        return fail(c, DASH_ERR_INVALID_ARG, "G, L, R must not overlap");
    HIP_TRY(c, hipSetDevice(c->device));
    GemmLaunch g;
    memset(&g, 0, sizeof(g));
    g.nprob = 1; g.B = Bm; g.nblocks = N; g.half = HALF_NONE;
    g.sym = c->symmetric ? 1 : 0;       // G G^T and G^T G are symmetric to the last bit
    // L = beta L + alpha G G^T : (Bm x Bn)(Bn x Bm)
    g.prob[0] = g.prob[1] = problem(G, G, L, L, nullptr, alpha, beta, 0.f, 0, 1);
    g.M = Bm; g.N = Bm; g.K = Bn;
    DASH_TRY(run_gemm(c, g));
    // R = beta R + alpha G^T G : (Bn x Bm)(Bm x Bn)
    g.prob[0] = g.prob[1] = problem(G, G, R, R, nullptr, alpha, beta, 0.f, 1, 0);
    g.M = Bn; g.N = Bn; g.K = Bm;
    DASH_TRY(run_gemm(c, g));
    return DASH_OK;
}

dash_status dash_precondition_rect(dash_ctx* c, const float* Linv, const float* G, const float* Rinv, float* U, int64_t N,
                                   int Bm, int Bn) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(Bm) || !valid_B(Bn))
        return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and Bm, Bn multiples of 64 (N=%lld Bm=%d Bn=%d)", (long long)N, Bm, Bn);
    if (N == 0) return DASH_OK;
    if (!Linv || !G || !Rinv || !U) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    const size_t gsz = (size_t)Bm * Bn;
    if (overlap2(U, (size_t)N * gsz * 4, G, (size_t)N * gsz * 4) || overlap2(U, (size_t)N * gsz * 4, Linv, (size_t)N * Bm * Bm * 4) ||
        overlap2(U, (size_t)N * gsz * 4, Rinv, (size_t)N * Bn * Bn * 4))
        return fail(c, DASH_ERR_INVALID_ARG, "U overlaps an input");
    HIP_TRY(c, hipSetDevice(c->device));
    const size_t per = gsz * sizeof(float);
    if (!c->ws || c->ws_bytes < per) return fail(c, DASH_ERR_WORKSPACE, "workspace holds %zu bytes, one block needs %zu", c->ws_bytes, per);
    int64_t chunk = (int64_t)(c->ws_bytes / per);
    if (chunk > N) chunk = N;
    float* T = (float*)c->ws;
    for (int64_t b0 = 0; b0 < N; b0 += chunk) {
        const int64_t nb = N - b0 < chunk ? N - b0 : chunk;
        GemmLaunch g;
        memset(&g, 0, sizeof(g));
        g.nprob = 1; g.B = Bm; g.nblocks = nb; g.half = HALF_NONE;
        // T = Linv G : (Bm x Bm)(Bm x Bn)
        g.prob[0] = g.prob[1] = problem(Linv + (size_t)b0 * Bm * Bm, G + (size_t)b0 * gsz, nullptr, T, nullptr, 1.f, 0.f, 0.f);
        g.M = Bm; g.N = Bn; g.K = Bm;
        DASH_TRY(run_gemm(c, g));
        // U = T Rinv : (Bm x Bn)(Bn x Bn)
        g.prob[0] = g.prob[1] = problem(T, Rinv + (size_t)b0 * Bn * Bn, nullptr, U + (size_t)b0 * gsz, nullptr, 1.f, 0.f, 0.f);
        g.M = Bm; g.N = Bn; g.K = Bn;
        DASH_TRY(run_gemm(c, g));
    }
    return DASH_OK;
}

// ---- block() and its inverse (Section 4.1) ----
static int64_t round_up(int64_t v, int64_t to) { return (v + to - 1) / to * to; }

static dash_status block_layer_impl(dash_ctx* c, float* W, int64_t m, int64_t n, int B, int pad_m, int pad_n,
                                    float* full, float* row_rest, float* col_rest, float* corner, bool scatter) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (m < 0 || n < 0 || B <= 0) return fail(c, DASH_ERR_INVALID_ARG, "need m, n >= 0 and B > 0 (m=%lld n=%lld B=%d)", (long long)m, (long long)n, B);
    if (pad_m < 1 || pad_n < 1 || B % pad_m || B % pad_n)
        return fail(c, DASH_ERR_INVALID_ARG, "the padding units must divide B (pad_m=%d pad_n=%d B=%d)", pad_m, pad_n, B);
    if (m == 0 || n == 0) return DASH_OK;
    const int64_t Nm = m / B, Nn = n / B;
    const int rm = (int)(m % B), rn = (int)(n % B);
    const int pm = (int)round_up(rm, pad_m), pn = (int)round_up(rn, pad_n);      // rest extents inside the stacks
    if (!W || (Nm * Nn > 0 && !full) || (rm && Nn && !row_rest) || (rn && Nm && !col_rest) || (rm && rn && !corner))
        return fail(c, DASH_ERR_INVALID_ARG, "null pointer for a non-empty group");
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, launch_block_copy(W, full, n, 0, 0, B, B, B, B, B, Nm, Nn, scatter, c->stream));
    if (rm) HIP_TRY(c, launch_block_copy(W, row_rest, n, Nm * B, 0, B, rm, B, pm, B, 1, Nn, scatter, c->stream));
    if (rn) HIP_TRY(c, launch_block_copy(W, col_rest, n, 0, Nn * B, B, B, rn, B, pn, Nm, 1, scatter, c->stream));
    if (rm && rn) HIP_TRY(c, launch_block_copy(W, corner, n, Nm * B, Nn * B, B, rm, rn, pm, pn, 1, 1, scatter, c->stream));
    return DASH_OK;
}

dash_status dash_block_layer(dash_ctx* c, const float* W, int64_t m, int64_t n, int B, float* full, float* row_rest,
                             float* col_rest, float* corner) {
    return block_layer_impl(c, const_cast<float*>(W), m, n, B, 1, 1, full, row_rest, col_rest, corner, false);
}

dash_status dash_unblock_layer(dash_ctx* c, float* W, int64_t m, int64_t n, int B, const float* full,
                               const float* row_rest, const float* col_rest, const float* corner) {
    return block_layer_impl(c, W, m, n, B, 1, 1, const_cast<float*>(full), const_cast<float*>(row_rest),
                            const_cast<float*>(col_rest), const_cast<float*>(corner), true);
}

dash_status dash_block_layer_padded(dash_ctx* c, const float* W, int64_t m, int64_t n, int B, int pad_m, int pad_n,
                                    float* full, float* row_rest, float* col_rest, float* corner) {
    return block_layer_impl(c, const_cast<float*>(W), m, n, B, pad_m, pad_n, full, row_rest, col_rest, corner, false);
}

dash_status dash_unblock_layer_padded(dash_ctx* c, float* W, int64_t m, int64_t n, int B, int pad_m, int pad_n,
                                      const float* full, const float* row_rest, const float* col_rest,
                                      const float* corner) {
    return block_layer_impl(c, W, m, n, B, pad_m, pad_n, const_cast<float*>(full), const_cast<float*>(row_rest),
                            const_cast<float*>(col_rest), const_cast<float*>(corner), true);
}

// ---- 1-D parameters (Section 4.1, normalisation layers): gradient blocks are vectors, only L exists ----
dash_status dash_accumulate_vector(dash_ctx* c, const float* g, float* L, int64_t N, int B, float beta, float alpha) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64");
    if (N == 0) return DASH_OK;
    if (!g || !L) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, launch_outer_accumulate(g, L, N, B, beta, alpha, c->stream));
    return DASH_OK;
}

dash_status dash_precondition_vector(dash_ctx* c, const float* Linv, const float* g, float* u, int64_t N, int B) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64");
    if (N == 0) return DASH_OK;
    if (!Linv || !g || !u) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    if (overlap(u, g, (size_t)N * B * 4) || overlap2(u, (size_t)N * B * 4, Linv, (size_t)N * B * B * 4))
        return fail(c, DASH_ERR_INVALID_ARG, "u overlaps an input");
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, launch_matvec(Linv, g, u, N, B, c->stream));
    return DASH_OK;
}

dash_status dash_block_norms(dash_ctx* c, const float* A, int64_t N, int B, float eps, dash_scaling scaling,
                             float* s_out) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64");
    if ((int)scaling < 0 || (int)scaling > 3) return fail(c, DASH_ERR_INVALID_ARG, "bad scaling");
    if (N == 0) return DASH_OK;
    if (!A || !s_out) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    HIP_TRY(c, hipSetDevice(c->device));
    const size_t per = scale_scratch_bytes(B), slack = 4 * WS_ALIGN * 16;
    if (!c->ws || c->ws_bytes < per + slack)
        return fail(c, DASH_ERR_WORKSPACE, "workspace holds %zu bytes, one block needs %zu", c->ws_bytes, per + slack);
    int64_t chunk = (int64_t)((c->ws_bytes - slack) / per);
    if (chunk > N) chunk = N;
    for (int64_t b0 = 0; b0 < N; b0 += chunk) {
        const int64_t nb = N - b0 < chunk ? N - b0 : chunk;
        Carve cv{c->ws, c->ws + c->ws_bytes};
        ScaleScratch sc;
        if (!sc.carve(cv, nb, B)) return fail(c, DASH_ERR_WORKSPACE, "internal: workspace carve failed");
        DASH_TRY(compute_scales(c, A + (size_t)b0 * B * B, nb, B, eps, scaling, 2, sc, s_out + b0));
    }
    return DASH_OK;
}

dash_status dash_block_norms_static(dash_ctx* c, const float* A, int64_t N, int B, float eps, dash_scaling scaling,
                                    float* s_out) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64");
    if (scaling == DASH_SCALE_POWER_ITERATION)
        return fail(c, DASH_ERR_UNSUPPORTED, "dash_block_norms_static: power-iteration scaling needs the pool vectors of "
                                             "a workspace; use dash_block_norms");
    if ((int)scaling < 0 || (int)scaling > 2) return fail(c, DASH_ERR_INVALID_ARG, "bad scaling");
    if (N > STATIC_MAX_BLOCKS)
        return fail(c, DASH_ERR_INVALID_ARG, "dash_block_norms_static: %lld blocks exceed the static scratch of %lld blocks; "
                                             "use dash_block_norms with a workspace", (long long)N, (long long)STATIC_MAX_BLOCKS);
    if (N == 0) return DASH_OK;
    if (!A || !s_out) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    if (!c->static_scratch) return fail(c, DASH_ERR_HIP, "static scratch address was not resolved");
    HIP_TRY(c, hipSetDevice(c->device));
    static_assert(STATIC_SLABS >= 32, "norm_slabs(B) is at most 32");
    float* partial = c->static_scratch;        // every partial a finalize reads is written by this call first
    if (scaling != DASH_SCALE_NONE) HIP_TRY(c, launch_norm_partials(A, N, B, eps, (int)scaling, partial, c->stream));
    HIP_TRY(c, launch_finalize_scale(partial, N, norm_slabs(B), (int)scaling, 2, s_out, nullptr, nullptr, c->stream));
    return DASH_OK;
}

dash_status dash_chebyshev_fit(int p, int degree, double a, double b, int n_points, double* coeffs_out) {
    if ((p != 2 && p != 4) || degree < 0 || n_points < degree + 1 || !(b > a) || !(a > 0.0) || !coeffs_out)
        return DASH_ERR_INVALID_ARG;
    // Appendix A.1: c_k = (w_k / N) sum_v f(x_v) T_k(t_v) over the N roots t_v of T_N, w_0 = 1, w_k = 2.
    // One pass over the nodes; at each node all T_k(t_v) come from the three-term recurrence
    // T_{k+1} = 2 t T_k - T_{k-1} (no cosine per coefficient), and node v adds f(x_v) T_k(t_v) to every sum.
    const double pi = 3.14159265358979323846;
    std::vector<double> sum((size_t)degree + 1, 0.0);
    for (int v = 0; v < n_points; ++v) {
        const double t = std::cos((v + 0.5) * pi / n_points);
        const double fx = std::pow(a + 0.5 * (b - a) * (1.0 + t), -1.0 / p);
        double t_prev = 1.0, t_cur = t;                      // T_0, T_1
        sum[0] += fx;
        if (degree >= 1) sum[1] += fx * t;
        for (int k = 2; k <= degree; ++k) {
            const double t_next = 2.0 * t * t_cur - t_prev;
            sum[(size_t)k] += fx * t_next;
            t_prev = t_cur;
            t_cur = t_next;
        }
    }
    for (int k = 0; k <= degree; ++k) coeffs_out[k] = sum[(size_t)k] * (k == 0 ? 1.0 : 2.0) / n_points;
    return DASH_OK;
}

dash_status dash_inverse_root(dash_ctx* c, const float* A, float* X, int64_t N, int B, dash_method method, int p,
                              int iters, float eps, dash_scaling scaling, dash_precision precision,
                              const double* cheb_coeffs, double cheb_a, double cheb_b, float* scale_out,
                              int32_t* nonfinite_out) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64 (N=%lld B=%d)", (long long)N, B);
    if (p != 2 && p != 4) return fail(c, DASH_ERR_INVALID_ARG, "p must be 2 or 4 (got %d)", p);
    if (method != DASH_NEWTON_DB && method != DASH_CHEBYSHEV && method != DASH_COUPLED_NEWTON)
        return fail(c, DASH_ERR_INVALID_ARG, "bad method");
    if (method == DASH_COUPLED_NEWTON && iters < 1) return fail(c, DASH_ERR_INVALID_ARG, "Coupled-Newton needs iters >= 1");
    if ((int)scaling < 0 || (int)scaling > 3) return fail(c, DASH_ERR_INVALID_ARG, "bad scaling");
    if (precision != DASH_FP32 && precision != DASH_BF16_ACC32 && precision != DASH_FP16_ACC32 && precision != DASH_BF16X3 &&
        precision != DASH_BF16X6 && precision != DASH_FP16X3)
        return fail(c, DASH_ERR_INVALID_ARG, "bad precision");
    c->half_kind = (precision == DASH_FP16_ACC32 || precision == DASH_FP16X3) ? HALF_FP16 : HALF_BF16;
    if (method == DASH_NEWTON_DB && iters < 1) return fail(c, DASH_ERR_INVALID_ARG, "Newton-DB needs iters >= 1");
    if (method == DASH_CHEBYSHEV) {
        if (iters < 2) return fail(c, DASH_ERR_INVALID_ARG, "Chebyshev needs degree >= 2");
        if (!cheb_coeffs) return fail(c, DASH_ERR_INVALID_ARG, "Chebyshev needs coefficients");
        if (!(cheb_b > cheb_a)) return fail(c, DASH_ERR_INVALID_ARG, "Chebyshev interval must have b > a");
    }
    if (!(eps >= 0.f)) return fail(c, DASH_ERR_INVALID_ARG, "eps must be >= 0");
    if (N == 0) return DASH_OK;
    if (!A || !X) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    if (overlap(A, X, (size_t)N * B * B * sizeof(float))) return fail(c, DASH_ERR_INVALID_ARG, "X overlaps A");
    HIP_TRY(c, hipSetDevice(c->device));

    const size_t per = per_block_bytes(B, method, precision);
    const size_t slack = 4 * WS_ALIGN * 16;
    if (!c->ws || c->ws_bytes < per + slack)
        return fail(c, DASH_ERR_WORKSPACE, "workspace holds %zu bytes, one block needs %zu", c->ws_bytes, per + slack);
    int64_t chunk = (int64_t)((c->ws_bytes - slack) / per);
    if (chunk > N) chunk = N;

    const size_t mat = (size_t)B * B;
    const int P = norm_slabs(B);
    const int nbuf = f32_buffers(method, precision), nhbuf = bf16_buffers(method, precision);
    const bool lowp = precision != DASH_FP32;
    const int planes = precision == DASH_BF16X6 ? 3 : (precision == DASH_BF16X3 || precision == DASH_FP16X3) ? 2 : 1;
    hipStream_t st = c->stream;

    for (int64_t b0 = 0; b0 < N; b0 += chunk) {
        const int64_t nb = N - b0 < chunk ? N - b0 : chunk;
        Carve cv{c->ws, c->ws + c->ws_bytes};
        ScaleScratch sc;
        const bool sc_ok = sc.carve(cv, nb, B);
        float* inv_s = sc.inv_s;
        float* unscale = sc.unscale;
        float* buf[9] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
        bf16_t* hbuf[27];
        for (int i = 0; i < 27; ++i) hbuf[i] = nullptr;
        for (int i = 0; i < nbuf; ++i) buf[i] = (float*)cv.take((size_t)nb * mat * sizeof(float));
        for (int i = 0; i < nhbuf; ++i) hbuf[i] = (bf16_t*)cv.take((size_t)nb * mat * sizeof(bf16_t));
        if (!sc_ok || (nbuf && !buf[nbuf - 1]) || (nhbuf && !hbuf[nhbuf - 1]))
            return fail(c, DASH_ERR_WORKSPACE, "internal: workspace carve failed");

        const float* Ac = A + (size_t)b0 * mat;
        float* Xc = X + (size_t)b0 * mat;
        int32_t* nf = nonfinite_out ? nonfinite_out + b0 : nullptr;
        if (nf) HIP_TRY(c, launch_fill_i32(nf, nb, 0, st));

        // Sections 3.4, 3.5: s = ||A + eps I||_F, trace, or 2 lambda_PI, kept with 1/s and s^(-1/p)
        DASH_TRY(compute_scales(c, Ac, nb, B, eps, scaling, p, sc, scale_out ? scale_out + b0 : sc.s));

        // small blocks: the iterative part of the chunk runs as two lanes on two streams (see dash_ctx::lanes)
        LaneScope lanes_of_chunk(c, chunk_takes_lanes(c, nb, B, precision) ? 2 : 1);
        DASH_TRY(lanes_of_chunk.fork());
        const dash_status chunk_status = [&]() -> dash_status {

        if (method == DASH_COUPLED_NEWTON && lowp) {
            DASH_TRY(cn_chunk_half(c, hbuf, Ac, Xc, nb, B, p, iters, eps, inv_s, unscale, nf, nullptr,
                                   planes >= 2 ? hbuf + 9 : nullptr, planes == 3 ? hbuf + 18 : nullptr));
        } else if (method == DASH_COUPLED_NEWTON) {
            DASH_TRY(cn_chunk(c, buf, Ac, Xc, nb, B, p, iters, eps, inv_s, unscale, nf));
        } else if (lowp && method == DASH_NEWTON_DB) {
            int idx = -1;
            bf16_t** lows = planes >= 2 ? hbuf + 5 : nullptr;      // low (middle) planes of the split modes
            bf16_t** lows2 = planes == 3 ? hbuf + 10 : nullptr;    // lowest planes of the three-plane mode
            if (p == 2) {
                DASH_TRY(ndb_call_bf16(c, hbuf, lows, lows2, buf[0], -1, nb, B, iters, false, true, Ac, eps, inv_s, Xc, unscale, nf, &idx));
            } else {
                DASH_TRY(ndb_call_bf16(c, hbuf, lows, lows2, buf[0], -1, nb, B, iters, true, true, Ac, eps, inv_s, nullptr, nullptr, nullptr, &idx));
                int idx2 = -1;
                DASH_TRY(ndb_call_bf16(c, hbuf, lows, lows2, buf[0], idx, nb, B, iters, false, false, nullptr, 0.f, nullptr, Xc, unscale, nf, &idx2));
            }
        } else if (lowp) {
            DASH_TRY(clenshaw_chunk_bf16(c, buf, hbuf, Ac, Xc, nb, B, iters, cheb_coeffs, cheb_a, cheb_b, eps, inv_s, unscale, nf,
                                         planes >= 2 ? hbuf + 3 : nullptr, planes == 3 ? hbuf + 6 : nullptr));
        } else if (method == DASH_NEWTON_DB) {
            int idx = -1;
            if (p == 2) {
                DASH_TRY(ndb_call(c, buf, -1, nb, B, iters, false, true, Ac, eps, inv_s, Xc, unscale, nf, &idx));
            } else {
                DASH_TRY(ndb_call(c, buf, -1, nb, B, iters, true, true, Ac, eps, inv_s, nullptr, nullptr, nullptr, &idx));
                int idx2 = -1;
                DASH_TRY(ndb_call(c, buf, idx, nb, B, iters, false, false, nullptr, 0.f, nullptr, Xc, unscale, nf, &idx2));
            }
        } else {
            DASH_TRY(clenshaw_chunk(c, buf, Ac, Xc, nb, B, iters, cheb_coeffs, cheb_a, cheb_b, eps, inv_s, unscale, nf));
        }
        return DASH_OK;
        }();
        const dash_status join_status = lanes_of_chunk.join();       // joined also when a launch of the chunk failed
        if (chunk_status != DASH_OK) return chunk_status;
        DASH_TRY(join_status);
    }
    return DASH_OK;
}

dash_status dash_precondition(dash_ctx* c, const float* Linv, const float* G, const float* Rinv, float* U, int64_t N,
                              int B) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64 (N=%lld B=%d)", (long long)N, B);
    if (N == 0) return DASH_OK;
    if (!Linv || !G || !Rinv || !U) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    const size_t mat = (size_t)B * B, bytes = (size_t)N * mat * sizeof(float);
    if (overlap(U, Linv, bytes) || overlap(U, G, bytes) || overlap(U, Rinv, bytes))
        return fail(c, DASH_ERR_INVALID_ARG, "U overlaps an input");
    HIP_TRY(c, hipSetDevice(c->device));
    const size_t per = mat * sizeof(float);
    if (!c->ws || c->ws_bytes < per) return fail(c, DASH_ERR_WORKSPACE, "workspace holds %zu bytes, one block needs %zu", c->ws_bytes, per);
    int64_t chunk = (int64_t)(c->ws_bytes / per);
    if (chunk > N) chunk = N;
    float* T = (float*)c->ws;
    for (int64_t b0 = 0; b0 < N; b0 += chunk) {
        const int64_t nb = N - b0 < chunk ? N - b0 : chunk;
        const size_t o = (size_t)b0 * mat;
        DASH_TRY(gemm1(c, problem(Linv + o, G + o, nullptr, T, nullptr, 1.f, 0.f, 0.f), nb, B));
        DASH_TRY(gemm1(c, problem(T, Rinv + o, nullptr, U + o, nullptr, 1.f, 0.f, 0.f), nb, B));
    }
    return DASH_OK;
}

dash_status dash_graft_update(dash_ctx* c, const float* G, const float* U, float* Acc, float* theta, int64_t N, int B,
                              float beta_g, float eps_g, float lr, float* s_out) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || !valid_B(B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64");
    if (N == 0) return DASH_OK;
    if (!G || !U || !Acc) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    HIP_TRY(c, hipSetDevice(c->device));
    const size_t per = SCALARS_PER_BLOCK;
    if (!c->ws || c->ws_bytes < per) return fail(c, DASH_ERR_WORKSPACE, "workspace needed (%zu bytes per block)", per);
    int64_t chunk = (int64_t)(c->ws_bytes / per);
    if (chunk > N) chunk = N;
    const size_t mat = (size_t)B * B;
    float* partial = (float*)c->ws;
    for (int64_t b0 = 0; b0 < N; b0 += chunk) {
        const int64_t nb = N - b0 < chunk ? N - b0 : chunk;
        const size_t o = (size_t)b0 * mat;
        HIP_TRY(c, launch_graft_partials(G + o, U + o, Acc + o, nb, (int64_t)mat, beta_g, eps_g, partial, c->stream));
        HIP_TRY(c, launch_graft_apply(U + o, theta ? theta + o : nullptr, partial, nb, (int64_t)mat, lr,
                                      s_out ? s_out + b0 : nullptr, nullptr, c->stream));
    }
    return DASH_OK;
}

dash_status dash_graft_scale(dash_ctx* c, const float* G, const float* U, float* Acc, int64_t N, int64_t elems,
                             float beta_g, float eps_g, float* U_scaled, float* s_out) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (N < 0 || elems <= 0 || elems % 4 || elems % (4 * graft_slabs(elems)))
        return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and the block size a multiple of 4 (of 32 from 4096, of 128 from 65536 on)");
    if (N == 0) return DASH_OK;
    if (!G || !U || !Acc) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    HIP_TRY(c, hipSetDevice(c->device));
    const size_t per = SCALARS_PER_BLOCK;
    if (!c->ws || c->ws_bytes < per) return fail(c, DASH_ERR_WORKSPACE, "workspace needed (%zu bytes per block)", per);
    int64_t chunk = (int64_t)(c->ws_bytes / per);
    if (chunk > N) chunk = N;
    float* partial = (float*)c->ws;
    for (int64_t b0 = 0; b0 < N; b0 += chunk) {
        const int64_t nb = N - b0 < chunk ? N - b0 : chunk;
        const size_t o = (size_t)b0 * elems;
        HIP_TRY(c, launch_graft_partials(G + o, U + o, Acc + o, nb, elems, beta_g, eps_g, partial, c->stream));
        HIP_TRY(c, launch_graft_apply(U + o, nullptr, partial, nb, elems, 0.f, s_out ? s_out + b0 : nullptr,
                                      U_scaled ? U_scaled + o : nullptr, c->stream));
    }
    return DASH_OK;
}

dash_status dash_apply_update(dash_ctx* c, float* theta, const float* update, int64_t n, float lr) {
    if (!c) return DASH_ERR_INVALID_ARG;
    if (n < 0) return fail(c, DASH_ERR_INVALID_ARG, "element count must not be negative");
    if (n == 0) return DASH_OK;
    if (!theta || !update) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    if (((uintptr_t)theta | (uintptr_t)update) % 16) return fail(c, DASH_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, launch_axpy(theta, update, n, lr, c->stream));
    return DASH_OK;
}

dash_status dash_step(dash_ctx* c, const dash_step_args* a) {
    if (!c || !a) return DASH_ERR_INVALID_ARG;
    if (a->N < 0 || !valid_B(a->B)) return fail(c, DASH_ERR_INVALID_ARG, "N must be >= 0 and B a multiple of 64");
    if (a->N == 0) return DASH_OK;
    if (!a->G || !a->S || !a->X || !a->U) return fail(c, DASH_ERR_INVALID_ARG, "null operand");
    if (a->graft && !a->graft_acc) return fail(c, DASH_ERR_INVALID_ARG, "grafting needs graft_acc");
    const size_t mat = (size_t)a->B * a->B;
    float* L = a->S;
    float* R = a->S + (size_t)a->N * mat;
    // Algorithm 1: EMA of the factors
    DASH_TRY(dash_accumulate_factors(c, a->G, L, R, a->N, a->B, a->beta, a->alpha));
    // roots of all 2N damped blocks in one call over the stack [L; R] (Section 4.1)
    if (a->refresh)
        DASH_TRY(dash_inverse_root(c, a->S, a->X, 2 * a->N, a->B, (dash_method)a->method, a->p, a->iters, a->eps,
                                   (dash_scaling)a->scaling, (dash_precision)a->precision, a->cheb_coeffs, a->cheb_a,
                                   a->cheb_b, nullptr, a->nonfinite_out));
    // Algorithm 1: U = L^{-1/p} G R^{-1/p}
    DASH_TRY(dash_precondition(c, a->X, a->G, a->X + (size_t)a->N * mat, a->U, a->N, a->B));
    if (a->graft)
        DASH_TRY(dash_graft_update(c, a->G, a->U, a->graft_acc, a->theta, a->N, a->B, a->beta_g, a->eps_g, a->lr, nullptr));
    return DASH_OK;
}

}  // extern "C"
