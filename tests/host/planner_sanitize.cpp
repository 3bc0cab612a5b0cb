// Host-side check of the model planner (csrc/model.hip compiled as plain C++ with the library calls stubbed):
// random models through create / describe / step under AddressSanitizer and UBSan.  Built and run by
// tests/test_host_sanitize.py; needs no GPU.
#include "dash.h"
#include <cstdio>
#include <cstdlib>
// stubs of the library calls the model layer makes (planning never calls them)
extern "C" {
const char* dash_last_error(const dash_ctx*) { return ""; }
size_t dash_workspace_bytes(int64_t n, int B, dash_method, int, dash_precision) { return (size_t)n * B * B * 20; }
dash_status dash_block_layer_padded(dash_ctx*, const float*, int64_t, int64_t, int, int, int, float*, float*, float*, float*) { return DASH_OK; }
dash_status dash_unblock_layer_padded(dash_ctx*, float*, int64_t, int64_t, int, int, int, const float*, const float*, const float*, const float*) { return DASH_OK; }
dash_status dash_accumulate_factors(dash_ctx*, const float*, float*, float*, int64_t, int, float, float) { return DASH_OK; }
dash_status dash_accumulate_factors_rect(dash_ctx*, const float*, float*, float*, int64_t, int, int, float, float) { return DASH_OK; }
dash_status dash_accumulate_vector(dash_ctx*, const float*, float*, int64_t, int, float, float) { return DASH_OK; }
dash_status dash_precondition(dash_ctx*, const float*, const float*, const float*, float*, int64_t, int) { return DASH_OK; }
dash_status dash_precondition_rect(dash_ctx*, const float*, const float*, const float*, float*, int64_t, int, int) { return DASH_OK; }
dash_status dash_precondition_vector(dash_ctx*, const float*, const float*, float*, int64_t, int) { return DASH_OK; }
dash_status dash_inverse_root(dash_ctx*, const float*, float*, int64_t, int, dash_method, int, int, float, dash_scaling, dash_precision, const double*, double, double, float*, int32_t*) { return DASH_OK; }
dash_status dash_graft_scale(dash_ctx*, const float*, const float*, float*, int64_t, int64_t, float, float, float*, float*) { return DASH_OK; }
dash_status dash_apply_update(dash_ctx*, float*, const float*, int64_t, float) { return DASH_OK; }
}
int main() {
    unsigned s = 1;
    for (int trial = 0; trial < 2000; ++trial) {
        int nl = 1 + (s = s * 1664525u + 1013904223u) % 12;
        dash_layer_shape L[12];
        int B = 64 * (1 + (s = s * 1664525u + 1013904223u) % 8);
        for (int i = 0; i < nl; ++i) {
            const int unit = (trial & 1) ? 1 + (s = s * 1664525u + 1013904223u) % 97 : 64;     // odd trials: any shape
            L[i].m = unit * (1 + (s = s * 1664525u + 1013904223u) % 40);
            L[i].n = ((s = s * 1664525u + 1013904223u) % 4 == 0) ? 0 : unit * (1 + (s = s * 1664525u + 1013904223u) % 40);
        }
        dash_model* m = nullptr;
        if (dash_model_create((dash_ctx*)0x10, L, nl, B, 4, 2, &m) != DASH_OK) { printf("create failed\n"); return 1; }
        dash_model_info info; dash_model_get_info(m, &info);
        int64_t blocks = 0;
        for (int i = 0; i < info.n_buckets; ++i) {
            int32_t bm, bn; int64_t c; dash_model_get_bucket(m, i, &bm, &bn, &c); blocks += c;
            if (bm <= 0 || bm % 64 || bn % 64 || bm > B || bn > B) { printf("bucket %d x %d\n", bm, bn); return 1; }    // padded to the kernels' granularity
        }
        if (blocks != info.n_gradient_blocks) { printf("count mismatch\n"); return 1; }
        // step through the whole sequence with a fake arena (stubs touch nothing)
        void* arena = aligned_alloc(256, 256);
        // arena too small must be refused
        if (info.arena_bytes > 256 && dash_model_set_arena(m, arena, 256) == DASH_OK) { printf("small arena accepted\n"); return 1; }
        free(arena);
        const float* g[12]; float* u[12];
        for (int i = 0; i < nl; ++i) { g[i] = (const float*)0x1000; u[i] = (float*)0x2000; }
        dash_model_set_arena(m, (void*)0x100000, (size_t)info.arena_bytes);
        dash_model_step_args a = {}; a.grads = g; a.updates = u; a.beta = 0.9f; a.alpha = 0.1f; a.eps = 1e-6f; a.iters = 5; a.refresh = 1; a.graft = 1;
        if (dash_model_step(m, &a) != DASH_OK) { printf("step failed: %s\n", dash_model_last_error(m)); return 1; }
        dash_model_destroy(m);
    }
    printf("sanitized planner ok\n");
    return 0;
}
