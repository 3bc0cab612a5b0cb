// Stacking across all layers a GPU owns (paper Section 4.1, the variant it calls DashGpu): the blocks
// of every layer are bucketed by shape, every factor of the same size -- whatever layer or side it
// belongs to -- sits in one stack, and one optimizer step issues one accumulate and one precondition
// per bucket and ONE inverse-root call per factor size.  Host-side planning plus a sequence of calls
// of the public entry points of dash.h; no kernels of its own.
#include "../../include/dash.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <new>
#include <tuple>
#include <vector>

namespace {

constexpr size_t ALIGN = 256;
size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct Bucket {                 // all gradient blocks of one shape
    int bm, bn;                 // vector buckets: bm entries, bn = 0
    int64_t count;
    int stackL, stackR;         // factor stacks holding its L and R segments (stackR = -1 for vectors)
    int64_t offL, offR;         // first block of the segment inside the stack
    size_t g_off, u_off;        // staging areas in the arena
    size_t acc_off;             // second-moment accumulator of the grafting (same shape as the staging)
};

struct Stack {                  // all factors of one size that take the same root
    int size, p;
    int64_t count;
    size_t s_off, x_off;
};

struct Part {                   // where one group of one layer lives: bucket and first block
    int bucket;
    int64_t first;
};

struct Layer {
    int64_t m, n;               // n = 0: 1-D parameter of m entries
    Part part[4];               // full, row rest, column rest, corner (bucket = -1: empty group)
};

}  // namespace

struct dash_model {
    dash_ctx* ctx;
    int B, p, p_vec;
    std::vector<Layer> layers;
    std::vector<Bucket> buckets;
    std::vector<Stack> stacks;
    size_t arena_bytes;
    char* arena;
    int64_t n_gradient_blocks, n_factor_blocks;
    char err[256];
};

namespace {

dash_status mfail(dash_model* m, dash_status st, const char* fmt, ...) {
    if (m) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(m->err, sizeof(m->err), fmt, ap);
        va_end(ap);
    }
    return st;
}

// error of a library call: keep the context's message
dash_status lib(dash_model* m, dash_status st) {
    if (st != DASH_OK && m->ctx) snprintf(m->err, sizeof(m->err), "%s", dash_last_error(m->ctx));
    return st;
}

float* at(const dash_model* m, size_t off) { return reinterpret_cast<float*>(m->arena + off); }

// rest extents are rounded up to the block-edge granularity of the product kernels; the padding is zero
constexpr int PAD = 64;
int64_t pad64(int64_t v) { return (v + PAD - 1) / PAD * PAD; }

}  // namespace

extern "C" {

dash_status dash_model_create(dash_ctx* ctx, const dash_layer_shape* layers, int n_layers, int B, int p, int p_vec,
                              dash_model** out) {
    if (!out) return DASH_ERR_INVALID_ARG;
    *out = nullptr;
    if ((!layers && n_layers > 0) || n_layers < 0 || B <= 0 || B % 64 || (p != 2 && p != 4) ||
        (p_vec != 2 && p_vec != 4))
        return DASH_ERR_INVALID_ARG;
    dash_model* m = new (std::nothrow) dash_model();
    if (!m) return DASH_ERR_INVALID_ARG;
    m->ctx = ctx; m->B = B; m->p = p; m->p_vec = p_vec; m->arena = nullptr; m->arena_bytes = 0; m->err[0] = 0;
    m->n_gradient_blocks = m->n_factor_blocks = 0;
    std::map<std::tuple<int, int>, int> bucket_of;           // (bm, bn) -> bucket
    auto place = [&](int bm, int bn, int64_t cnt) -> Part {
        if (cnt <= 0 || bm <= 0) return Part{-1, 0};
        auto key = std::make_tuple(bm, bn);
        auto it = bucket_of.find(key);
        if (it == bucket_of.end()) {
            it = bucket_of.emplace(key, (int)m->buckets.size()).first;
            m->buckets.push_back(Bucket{bm, bn, 0, -1, -1, 0, 0, 0, 0, 0});
        }
        Bucket& b = m->buckets[it->second];
        Part pt{it->second, b.count};
        b.count += cnt;
        return pt;
    };
    for (int l = 0; l < n_layers; ++l) {
        const int64_t mm = layers[l].m, nn = layers[l].n;
        Layer L;
        L.m = mm; L.n = nn;
        for (auto& pt : L.part) pt = Part{-1, 0};
        if (mm <= 0 || nn < 0) {
            delete m;
            return DASH_ERR_INVALID_ARG;
        }
        if (nn == 0) {          // 1-D: m / B vectors of B entries and one of m mod B
            const int64_t nv = mm / B;
            const int r = (int)pad64(mm % B);         // the remainder, zero padded to the next multiple of 64
            L.part[1] = place(B, 0, nv);
            L.part[3] = place(r, 0, r ? 1 : 0);
        } else {
            const int64_t Nm = mm / B, Nn = nn / B;
            const int rm = (int)pad64(mm % B), rn = (int)pad64(nn % B);     // rest extents inside the stacks
            L.part[0] = place(B, B, Nm * Nn);
            L.part[1] = place(rm, B, rm ? Nn : 0);
            L.part[2] = place(B, rn, rn ? Nm : 0);
            L.part[3] = place(rm, rn, (rm && rn) ? 1 : 0);
        }
        m->layers.push_back(L);
    }
    // factor stacks by (size, root)
    std::map<std::tuple<int, int>, int> stack_of;
    auto segment = [&](int size, int root, int64_t cnt, int* stack, int64_t* off) {
        auto key = std::make_tuple(size, root);
        auto it = stack_of.find(key);
        if (it == stack_of.end()) {
            it = stack_of.emplace(key, (int)m->stacks.size()).first;
            m->stacks.push_back(Stack{size, root, 0, 0, 0});
        }
        Stack& s = m->stacks[it->second];
        *stack = it->second;
        *off = s.count;
        s.count += cnt;
    };
    for (Bucket& b : m->buckets) {      // all left factors first, then the right ones
        segment(b.bm, b.bn ? p : p_vec, b.count, &b.stackL, &b.offL);
        m->n_gradient_blocks += b.count;
    }
    for (Bucket& b : m->buckets)
        if (b.bn) segment(b.bn, p, b.count, &b.stackR, &b.offR);
    size_t off = 0;
    for (Stack& s : m->stacks) {
        const size_t bytes = align_up((size_t)s.count * s.size * s.size * sizeof(float));
        s.s_off = off; off += bytes;
        s.x_off = off; off += bytes;
        m->n_factor_blocks += s.count;
    }
    for (Bucket& b : m->buckets) {
        const size_t bytes = align_up((size_t)b.count * b.bm * (b.bn ? b.bn : 1) * sizeof(float));
        b.g_off = off; off += bytes;
        b.u_off = off; off += bytes;
        b.acc_off = off; off += bytes;
    }
    m->arena_bytes = off;
    *out = m;
    return DASH_OK;
}

dash_status dash_model_destroy(dash_model* m) {
    delete m;
    return DASH_OK;
}

const char* dash_model_last_error(const dash_model* m) { return m ? m->err : "null model"; }

dash_status dash_model_get_info(const dash_model* m, dash_model_info* info) {
    if (!m || !info) return DASH_ERR_INVALID_ARG;
    info->n_layers = (int32_t)m->layers.size();
    info->n_buckets = (int32_t)m->buckets.size();
    info->n_stacks = (int32_t)m->stacks.size();
    info->B = m->B;
    info->n_gradient_blocks = m->n_gradient_blocks;
    info->n_factor_blocks = m->n_factor_blocks;
    info->arena_bytes = (int64_t)m->arena_bytes;
    return DASH_OK;
}

dash_status dash_model_get_bucket(const dash_model* m, int i, int32_t* bm, int32_t* bn, int64_t* count) {
    if (!m || i < 0 || i >= (int)m->buckets.size()) return DASH_ERR_INVALID_ARG;
    if (bm) *bm = m->buckets[i].bm;
    if (bn) *bn = m->buckets[i].bn;
    if (count) *count = m->buckets[i].count;
    return DASH_OK;
}

dash_status dash_model_get_stack(const dash_model* m, int i, int32_t* size, int32_t* p, int64_t* count, float** S,
                                 float** X) {
    if (!m || i < 0 || i >= (int)m->stacks.size()) return DASH_ERR_INVALID_ARG;
    const Stack& s = m->stacks[i];
    if (size) *size = s.size;
    if (p) *p = s.p;
    if (count) *count = s.count;
    if (S) *S = m->arena ? at(m, s.s_off) : nullptr;
    if (X) *X = m->arena ? at(m, s.x_off) : nullptr;
    return DASH_OK;
}

size_t dash_model_workspace_bytes(const dash_model* m, dash_method method, dash_precision precision) {
    if (!m) return 0;
    size_t need = 0;
    for (const Stack& s : m->stacks) {
        const size_t w = dash_workspace_bytes(s.count, s.size, method, s.p, precision);
        if (w > need) need = w;
    }
    for (const Bucket& b : m->buckets) {
        const size_t w = (size_t)b.count * b.bm * (b.bn ? b.bn : 1) * sizeof(float);
        if (w > need) need = w;
    }
    return need;
}

dash_status dash_model_set_arena(dash_model* m, void* dev_ptr, size_t bytes) {
    if (!m) return DASH_ERR_INVALID_ARG;
    if (dev_ptr && ((uintptr_t)dev_ptr % ALIGN)) return mfail(m, DASH_ERR_INVALID_ARG, "arena must be 256-byte aligned");
    if (dev_ptr && bytes < m->arena_bytes)
        return mfail(m, DASH_ERR_WORKSPACE, "arena holds %zu bytes, the model needs %zu", bytes, m->arena_bytes);
    m->arena = static_cast<char*>(dev_ptr);
    return DASH_OK;
}

dash_status dash_model_step(dash_model* m, const dash_model_step_args* a) {
    if (!m || !a) return DASH_ERR_INVALID_ARG;
    if (!m->ctx) return mfail(m, DASH_ERR_INVALID_ARG, "the model was created without a context (planning only)");
    if (!m->arena) return mfail(m, DASH_ERR_WORKSPACE, "no arena set");
    const int nl = (int)m->layers.size();
    if (nl && (!a->grads || !a->updates)) return mfail(m, DASH_ERR_INVALID_ARG, "null pointer array");
    for (int l = 0; l < nl; ++l)
        if (!a->grads[l] || !a->updates[l]) return mfail(m, DASH_ERR_INVALID_ARG, "layer %d: null gradient or update", l);
    dash_ctx* c = m->ctx;
    const int B = m->B;
    auto group = [&](const Layer& L, int g, bool upd) -> float* {       // staging of group g of a layer
        const Part& pt = L.part[g];
        if (pt.bucket < 0) return nullptr;
        const Bucket& b = m->buckets[pt.bucket];
        return at(m, upd ? b.u_off : b.g_off) + (size_t)pt.first * b.bm * (b.bn ? b.bn : 1);
    };
    // 1. block(): every layer's gradient into the staging stacks of its buckets.  A 1-D parameter of E
    //    entries is the 1 x E layer: its "row rest" are the E / B vectors, its "corner" the remainder.
    for (int l = 0; l < nl; ++l) {
        const Layer& L = m->layers[l];
        const int64_t mm = L.n ? L.m : 1, nn = L.n ? L.n : L.m;
        dash_status st = lib(m, dash_block_layer_padded(c, a->grads[l], mm, nn, B, L.n ? PAD : 1, PAD, group(L, 0, false),
                                                        group(L, 1, false), group(L, 2, false), group(L, 3, false)));
        if (st != DASH_OK) return st;
    }
    // 2. Kronecker factors, one call per bucket, written straight into the factor stacks
    for (const Bucket& b : m->buckets) {
        const Stack& sl = m->stacks[b.stackL];
        float* Lp = at(m, sl.s_off) + (size_t)b.offL * b.bm * b.bm;
        dash_status st;
        if (!b.bn) {
            st = dash_accumulate_vector(c, at(m, b.g_off), Lp, b.count, b.bm, a->beta, a->alpha);
        } else {
            const Stack& sr = m->stacks[b.stackR];
            float* Rp = at(m, sr.s_off) + (size_t)b.offR * b.bn * b.bn;
            st = b.bm == b.bn ? dash_accumulate_factors(c, at(m, b.g_off), Lp, Rp, b.count, b.bm, a->beta, a->alpha)
                              : dash_accumulate_factors_rect(c, at(m, b.g_off), Lp, Rp, b.count, b.bm, b.bn, a->beta, a->alpha);
        }
        if (lib(m, st) != DASH_OK) return st;
    }
    // 3. inverse roots: one call per factor size (skipped between refreshes: the stored roots are reused)
    if (a->refresh) {
        int64_t flag_off = 0;
        for (const Stack& s : m->stacks) {
            dash_status st = lib(m, dash_inverse_root(c, at(m, s.s_off), at(m, s.x_off), s.count, s.size,
                                                      (dash_method)a->method, s.p, a->iters, a->eps,
                                                      (dash_scaling)a->scaling, (dash_precision)a->precision,
                                                      a->cheb_coeffs, a->cheb_a, a->cheb_b, nullptr,
                                                      a->nonfinite_out ? a->nonfinite_out + flag_off : nullptr));
            if (st != DASH_OK) return st;
            flag_off += s.count;
        }
    }
    // 4. update directions per bucket
    for (const Bucket& b : m->buckets) {
        const Stack& sl = m->stacks[b.stackL];
        const float* Xl = at(m, sl.x_off) + (size_t)b.offL * b.bm * b.bm;
        dash_status st;
        if (!b.bn) {
            st = dash_precondition_vector(c, Xl, at(m, b.g_off), at(m, b.u_off), b.count, b.bm);
        } else {
            const Stack& sr = m->stacks[b.stackR];
            const float* Xr = at(m, sr.x_off) + (size_t)b.offR * b.bn * b.bn;
            st = b.bm == b.bn ? dash_precondition(c, Xl, at(m, b.g_off), Xr, at(m, b.u_off), b.count, b.bm)
                              : dash_precondition_rect(c, Xl, at(m, b.g_off), Xr, at(m, b.u_off), b.count, b.bm, b.bn);
        }
        if (lib(m, st) != DASH_OK) return st;
    }
    // 4b. block-wise Adam grafting (Section 2.3): U_b <- s_b U_b with s_b = ||P_b||_F / ||U_b||_F
    if (a->graft) {
        for (const Bucket& b : m->buckets) {
            const int64_t elems = (int64_t)b.bm * (b.bn ? b.bn : 1);
            dash_status st = lib(m, dash_graft_scale(c, at(m, b.g_off), at(m, b.u_off), at(m, b.acc_off), b.count, elems,
                                                     a->beta_g, a->eps_g, at(m, b.u_off), nullptr));
            if (st != DASH_OK) return st;
        }
    }
    // 5. back to the layers' own layout
    for (int l = 0; l < nl; ++l) {
        const Layer& L = m->layers[l];
        const int64_t mm = L.n ? L.m : 1, nn = L.n ? L.n : L.m;
        dash_status st = lib(m, dash_unblock_layer_padded(c, a->updates[l], mm, nn, B, L.n ? PAD : 1, PAD, group(L, 0, true),
                                                          group(L, 1, true), group(L, 2, true), group(L, 3, true)));
        if (st != DASH_OK) return st;
        // Algorithm 1, parameter update
        if (a->thetas && a->thetas[l]) {
            st = lib(m, dash_apply_update(c, a->thetas[l], a->updates[l], L.m * (L.n ? L.n : 1), a->lr));
            if (st != DASH_OK) return st;
        }
    }
    return DASH_OK;
}

}  // extern "C"
