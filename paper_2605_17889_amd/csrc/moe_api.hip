// C-ABI entry points of libmoe: argument validation, workspace, stage sequencing and the
// optional per-stage event timing. All arithmetic lives in the kernels of the other files.
#include <new>
#include <vector>

#include "common.h"

struct moe_ctx {
    moe_shape shape;
    int device;
    moe::GemmEnv gemm;   // device + tuning knobs of moe_set_gemm_config
    // workspace (device)
    unsigned char* base;
    size_t bytes;
    int32_t* topk_idx;   // [T_max, k]
    float* topk_w;       // [T_max, k]
    int32_t* counts;     // [E]
    int32_t* offsets;    // [E+1]
    int32_t* perm;       // [R_max]
    int32_t* inv_perm;   // [R_max]
    int32_t* scratch;    // permutation segment tables
    float* logits;       // [T_max, E] router logits, only with more than 16 experts (else null)
    moe_bf16* x_perm;    // [R_max, d]
    moe_bf16* H;         // [R_max, f]
    moe_bf16* y_perm;    // [R_max, d]
    float* y_perm_f32;   // [R_max, d], allocated by moe_set_expert_output_fp32; null = keep bf16
    // profiling
    bool prof_armed;
    int prof_max_calls, prof_calls;
    std::vector<hipEvent_t> prof_events;       // per recorded interval: start, stop
    std::vector<int> prof_stage;               // stage of each interval
    std::vector<int> prof_call;                // armed call (0-based) that the interval belongs to
    int64_t prof_launches[MOE_NUM_STAGES];
    // streamed experts (created by the first moe_layer_forward_streamed call, kept until destroy)
    hipStream_t copy_stream;
    unsigned char* slot[2];     // device staging, each W1_e | W3_e | W2_e of one expert
    hipEvent_t ready[2];        // recorded on copy_stream: the slot holds its expert
    hipEvent_t freed[2];        // recorded on the caller's stream: the slot's GEMMs are enqueued
    bool freed_valid[2];
};

namespace {

using namespace moe;

bool shape_ok(const moe_shape* s) {
    if (!s) return false;
    if (s->T_max < 0 || s->d_model <= 0 || s->d_ff <= 0 || s->E <= 0 || s->k <= 0) return false;
    if (s->d_model % 512 != 0 || s->d_ff % 128 != 0) return false;
    if (s->E > kMaxExperts || s->k > s->E || s->k > kWave) return false;
    if (static_cast<long long>(s->T_max) * s->k >= (1LL << 31)) return false;
    return true;
}

size_t align_up(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

// Kernels launch on the calling thread's current device: it must be the context's.
bool on_own_device(const moe_ctx* c) {
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess && dev == c->device;
}

struct Layout {
    size_t topk_idx, topk_w, counts, offsets, perm, inv_perm, scratch, logits, x_perm, H, y_perm, total;
};

Layout layout_for(const moe_shape* s) {
    Layout L{};
    const size_t T = static_cast<size_t>(s->T_max), R = T * s->k;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes); return at; };
    L.topk_idx = take(R * 4);
    L.topk_w = take(R * 4);
    L.counts = take(static_cast<size_t>(s->E) * 4);
    L.offsets = take(static_cast<size_t>(s->E + 1) * 4);
    L.perm = take(R * 4);
    L.inv_perm = take(R * 4);
    L.scratch = take(permute_scratch_ints(static_cast<int>(R), s->E) * 4);
    L.logits = take(s->E > 16 ? T * s->E * 4 : 0);
    L.x_perm = take(R * s->d_model * 2);
    L.H = take(R * s->d_ff * 2);
    L.y_perm = take(R * s->d_model * 2);
    L.total = off ? off : 256;
    return L;
}

// Stage timing: records a start/stop event pair around `fn` when armed.
template <typename Fn>
int run_stage(moe_ctx* c, int stage, int launches, hipStream_t s, Fn&& fn) {
    const bool rec = c->prof_armed && c->prof_calls <= c->prof_max_calls;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (rec) {
        MOE_HIP_TRY(hipEventCreate(&e0));
        MOE_HIP_TRY(hipEventCreate(&e1));
        MOE_HIP_TRY(hipEventRecord(e0, s));
    }
    const int rc = fn();
    if (rec) {
        MOE_HIP_TRY(hipEventRecord(e1, s));
        c->prof_events.push_back(e0);
        c->prof_events.push_back(e1);
        c->prof_stage.push_back(stage);
        c->prof_call.push_back(c->prof_calls - 1);
        c->prof_launches[stage] += launches;
    }
    return rc;
}

// Where the layer calls keep the expert outputs Yp between the down projection and the combine.
void* expert_out(moe_ctx* c) {
    return c->y_perm_f32 ? static_cast<void*>(c->y_perm_f32) : static_cast<void*>(c->y_perm);
}

int forward_chunk(moe_ctx* c, const moe_bf16* x, const float* w_router, const float* bias,
                  const moe_bf16* W1, const moe_bf16* W3, const moe_bf16* W2, int T, moe_bf16* y,
                  hipStream_t s) {
    const moe_shape& sh = c->shape;
    const int d = sh.d_model, f = sh.d_ff, E = sh.E, k = sh.k, R = T * k;
    int rc;
    rc = run_stage(c, MOE_STAGE_ROUTE, 1, s, [&] {
        return launch_route(x, w_router, bias, T, d, E, k, c->topk_idx, c->topk_w, nullptr, c->logits, s);
    });
    if (rc != MOE_OK) return rc;
    rc = run_stage(c, MOE_STAGE_PERMUTE, permute_launches(R), s, [&] {
        return launch_permute(c->topk_idx, R, E, c->counts, c->offsets, c->perm, c->inv_perm,
                              c->scratch, s);
    });
    if (rc != MOE_OK) return rc;
    // The row gather x -> x_perm is fused into the gate/up kernel's operand loads (it reads
    // token row perm[p] / k directly) whenever a token row's byte offset fits 32 bits.
    const bool fuse_gather =
        !c->gemm.materialise_gather && static_cast<unsigned long long>(T) * d * 2ull < (1ull << 32);
    if (!fuse_gather) {
        rc = run_stage(c, MOE_STAGE_GATHER, 1, s, [&] {
            return launch_gather(x, c->perm, c->offsets, R, d, k, E, c->x_perm, s);
        });
        if (rc != MOE_OK) return rc;
    }
    rc = run_stage(c, MOE_STAGE_GATEUP, 1, s, [&] {
        return fuse_gather
                   ? launch_gateup(c->gemm, x, c->perm, k, c->offsets, R, R, d, f, E, W1, W3, c->H, s)
                   : launch_gateup(c->gemm, c->x_perm, nullptr, 1, c->offsets, R, R, d, f, E, W1, W3, c->H, s);
    });
    if (rc != MOE_OK) return rc;
    rc = run_stage(c, MOE_STAGE_DOWN, 1, s, [&] {
        return launch_down(c->gemm, c->H, c->offsets, R, R, d, f, E, W2, expert_out(c), c->y_perm_f32 != nullptr, s);
    });
    if (rc != MOE_OK) return rc;
    return run_stage(c, MOE_STAGE_COMBINE, 1, s, [&] {
        return launch_combine(expert_out(c), c->y_perm_f32 != nullptr, c->inv_perm, c->topk_w, T, d, k, y, s);
    });
}

int ensure_streaming(moe_ctx* c) {
    if (c->copy_stream) return MOE_OK;
    const size_t bytes = static_cast<size_t>(3) * c->shape.d_model * c->shape.d_ff * sizeof(moe_bf16);
    void* p = nullptr;
    hipStream_t st = nullptr;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    int made = 0;
    int rc = MOE_OK;
    if (hipMalloc(&p, 2 * bytes) != hipSuccess) {
        (void)hipGetLastError();
        return MOE_ERR_WORKSPACE;
    }
    for (; made < 4; ++made)
        if (hipEventCreateWithFlags(&ev[made], hipEventDisableTiming) != hipSuccess) { rc = MOE_ERR_HIP; break; }
    if (rc == MOE_OK && hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess)   // default priority
        rc = MOE_ERR_HIP;
    if (rc != MOE_OK) {                       // leave the context as it was
        for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
        (void)hipFree(p);
        (void)hipGetLastError();
        return rc;
    }
    c->slot[0] = static_cast<unsigned char*>(p);
    c->slot[1] = c->slot[0] + bytes;
    for (int i = 0; i < 2; ++i) {
        c->ready[i] = ev[i];
        c->freed[i] = ev[2 + i];
        c->freed_valid[i] = false;
    }
    c->copy_stream = st;
    return MOE_OK;
}

}  // namespace

extern "C" {

const char* moe_status_string(int status) {
    switch (status) {
        case MOE_OK: return "MOE_OK";
        case MOE_ERR_INVALID_ARG: return "MOE_ERR_INVALID_ARG";
        case MOE_ERR_UNSUPPORTED_SHAPE: return "MOE_ERR_UNSUPPORTED_SHAPE";
        case MOE_ERR_WORKSPACE: return "MOE_ERR_WORKSPACE";
        case MOE_ERR_HIP: return "MOE_ERR_HIP";
        default: return "MOE_ERR_UNKNOWN";
    }
}

size_t moe_workspace_bytes(const moe_shape* shape) {
    if (!shape_ok(shape)) return 0;
    return layout_for(shape).total;
}

int moe_create(moe_ctx** out, const moe_shape* shape, int device_id) {
    if (!out) return MOE_ERR_INVALID_ARG;
    *out = nullptr;
    if (!shape) return MOE_ERR_INVALID_ARG;
    if (!shape_ok(shape)) return MOE_ERR_UNSUPPORTED_SHAPE;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess) return MOE_ERR_HIP;
    if (device_id < 0 || device_id >= ndev) return MOE_ERR_INVALID_ARG;
    if (device_id >= 64) return MOE_ERR_INVALID_ARG;
    int caller_device = 0;
    MOE_HIP_TRY(hipGetDevice(&caller_device));
    moe_ctx* c = new (std::nothrow) moe_ctx();
    if (!c) return MOE_ERR_WORKSPACE;
    c->shape = *shape;
    c->device = device_id;
    c->gemm.device = device_id;
    const Layout L = layout_for(shape);
    c->bytes = L.total;
    void* p = nullptr;
    // allocate on the context's device, then give the caller its current device back
    hipError_t err = hipSetDevice(device_id);
    if (err == hipSuccess) err = hipMalloc(&p, L.total);
    const hipError_t back = hipSetDevice(caller_device);
    if (err != hipSuccess || back != hipSuccess) {
        (void)hipGetLastError();
        if (p) (void)hipFree(p);
        delete c;
        return err != hipSuccess && back == hipSuccess ? MOE_ERR_WORKSPACE : MOE_ERR_HIP;
    }
    c->base = static_cast<unsigned char*>(p);
    c->topk_idx = reinterpret_cast<int32_t*>(c->base + L.topk_idx);
    c->topk_w = reinterpret_cast<float*>(c->base + L.topk_w);
    c->counts = reinterpret_cast<int32_t*>(c->base + L.counts);
    c->offsets = reinterpret_cast<int32_t*>(c->base + L.offsets);
    c->perm = reinterpret_cast<int32_t*>(c->base + L.perm);
    c->inv_perm = reinterpret_cast<int32_t*>(c->base + L.inv_perm);
    c->scratch = reinterpret_cast<int32_t*>(c->base + L.scratch);
    c->logits = shape->E > 16 ? reinterpret_cast<float*>(c->base + L.logits) : nullptr;
    c->x_perm = reinterpret_cast<moe_bf16*>(c->base + L.x_perm);
    c->H = reinterpret_cast<moe_bf16*>(c->base + L.H);
    c->y_perm = reinterpret_cast<moe_bf16*>(c->base + L.y_perm);
    c->y_perm_f32 = nullptr;
    c->prof_armed = false;
    c->prof_max_calls = c->prof_calls = 0;
    for (auto& v : c->prof_launches) v = 0;
    c->copy_stream = nullptr;
    c->slot[0] = c->slot[1] = nullptr;
    *out = c;
    return MOE_OK;
}

int moe_destroy(moe_ctx* c) {
    if (!c) return MOE_ERR_INVALID_ARG;
    for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
    int rc = MOE_OK;
    if (c->copy_stream) {
        if (hipStreamSynchronize(c->copy_stream) != hipSuccess) rc = MOE_ERR_HIP;
        (void)hipStreamDestroy(c->copy_stream);
        for (int i = 0; i < 2; ++i) {
            (void)hipEventDestroy(c->ready[i]);
            (void)hipEventDestroy(c->freed[i]);
        }
    }
    if (c->slot[0] && hipFree(c->slot[0]) != hipSuccess) rc = MOE_ERR_HIP;
    if (c->y_perm_f32 && hipFree(c->y_perm_f32) != hipSuccess) rc = MOE_ERR_HIP;
    if (c->base && hipFree(c->base) != hipSuccess) rc = MOE_ERR_HIP;
    delete c;
    return rc;
}

int moe_route(moe_ctx* c, const moe_bf16* x, const float* w_router, const float* bias, int32_t T,
              int32_t* topk_idx, float* topk_w, float* logits_out, void* stream) {
    if (!c || T < 0 || T > c->shape.T_max) return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!x || !w_router || !topk_idx || !topk_w) return MOE_ERR_INVALID_ARG;
    return launch_route(x, w_router, bias, T, c->shape.d_model, c->shape.E, c->shape.k, topk_idx,
                        topk_w, logits_out, c->logits, static_cast<hipStream_t>(stream));
}

int moe_route_from_logits(moe_ctx* c, const float* logits, int32_t T, int32_t* topk_idx,
                          float* topk_w, void* stream) {
    if (!c || T < 0 || T > c->shape.T_max) return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!logits || !topk_idx || !topk_w) return MOE_ERR_INVALID_ARG;
    return launch_route_from_logits(logits, T, c->shape.E, c->shape.k, topk_idx, topk_w,
                                    static_cast<hipStream_t>(stream));
}

int moe_permute(moe_ctx* c, const int32_t* topk_idx, int32_t T, int32_t* counts, int32_t* offsets,
                int32_t* perm, int32_t* inv_perm, const moe_bf16* x, moe_bf16* x_perm,
                void* stream) {
    if (!c || T < 0 || T > c->shape.T_max) return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    if (!counts || !offsets) return MOE_ERR_INVALID_ARG;
    if (T > 0 && (!topk_idx || !perm || !inv_perm)) return MOE_ERR_INVALID_ARG;
    if ((x == nullptr) != (x_perm == nullptr)) return MOE_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int R = T * c->shape.k;
    int rc = launch_permute(topk_idx, R, c->shape.E, counts, offsets, perm, inv_perm, c->scratch, s);
    if (rc != MOE_OK) return rc;
    if (x && T > 0)
        rc = launch_gather(x, perm, offsets, R, c->shape.d_model, c->shape.k, c->shape.E, x_perm, s);
    return rc;
}

int moe_expert_ffn(moe_ctx* c, const moe_bf16* x_perm, const int32_t* offsets, int32_t R,
                   const moe_bf16* W1, const moe_bf16* W3, const moe_bf16* W2, moe_bf16* y_perm,
                   void* stream) {
    if (!c || R < 0 || static_cast<long long>(R) > static_cast<long long>(c->shape.T_max) * c->shape.k)
        return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    if (R == 0) return MOE_OK;
    if (!x_perm || !offsets || !W1 || !W3 || !W2 || !y_perm) return MOE_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const moe_shape& sh = c->shape;
    if (c->prof_armed) ++c->prof_calls;
    int rc = run_stage(c, MOE_STAGE_GATEUP, 1, s, [&] {
        return launch_gateup(c->gemm, x_perm, nullptr, 1, offsets, R, R, sh.d_model, sh.d_ff, sh.E, W1, W3, c->H, s);
    });
    if (rc != MOE_OK) return rc;
    return run_stage(c, MOE_STAGE_DOWN, 1, s, [&] {
        return launch_down(c->gemm, c->H, offsets, R, R, sh.d_model, sh.d_ff, sh.E, W2, y_perm, false, s);
    });
}

int moe_combine(moe_ctx* c, const moe_bf16* y_perm, const int32_t* inv_perm, const float* topk_w,
                int32_t T, moe_bf16* y, void* stream) {
    if (!c || T < 0 || T > c->shape.T_max) return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!y_perm || !inv_perm || !topk_w || !y) return MOE_ERR_INVALID_ARG;
    return launch_combine(y_perm, false, inv_perm, topk_w, T, c->shape.d_model, c->shape.k, y,
                          static_cast<hipStream_t>(stream));
}

int moe_layer_forward(moe_ctx* c, const moe_bf16* x, const float* w_router, const float* bias,
                      const moe_bf16* W1, const moe_bf16* W3, const moe_bf16* W2, int32_t T,
                      moe_bf16* y, void* stream) {
    if (!c || T < 0 || T > c->shape.T_max) return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!x || !w_router || !W1 || !W3 || !W2 || !y) return MOE_ERR_INVALID_ARG;
    if (c->prof_armed) c->prof_calls++;
    return forward_chunk(c, x, w_router, bias, W1, W3, W2, T, y, static_cast<hipStream_t>(stream));
}

int moe_layer_forward_microbatched(moe_ctx* c, const moe_bf16* x, const float* w_router,
                                   const float* bias, const moe_bf16* W1, const moe_bf16* W3,
                                   const moe_bf16* W2, int32_t T, int32_t micro_tokens,
                                   moe_bf16* y, void* stream) {
    if (!c || T < 0 || T > c->shape.T_max || micro_tokens < 1) return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!x || !w_router || !W1 || !W3 || !W2 || !y) return MOE_ERR_INVALID_ARG;
    if (c->prof_armed) c->prof_calls++;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t d = static_cast<size_t>(c->shape.d_model);
    for (int t0 = 0; t0 < T; t0 += micro_tokens) {
        const int Tc = (T - t0 < micro_tokens) ? T - t0 : micro_tokens;
        const int rc = forward_chunk(c, x + t0 * d, w_router, bias, W1, W3, W2, Tc, y + t0 * d, s);
        if (rc != MOE_OK) return rc;
    }
    return MOE_OK;
}

int moe_layer_forward_streamed(moe_ctx* c, const moe_bf16* x, const float* w_router,
                               const float* bias, const moe_bf16* W1, const moe_bf16* W3,
                               const moe_bf16* W2, const moe_bf16* W1_host,
                               const moe_bf16* W3_host, const moe_bf16* W2_host,
                               int32_t n_streamed, int32_t T, moe_bf16* y, void* stream) {
    if (!c || T < 0 || T > c->shape.T_max || n_streamed < 0 || n_streamed > c->shape.E)
        return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    const moe_shape& sh = c->shape;
    const int d = sh.d_model, f = sh.d_ff, E = sh.E, k = sh.k, R = T * k;
    const int E_res = E - n_streamed;
    if (!x || !w_router || !y) return MOE_ERR_INVALID_ARG;
    if (E_res > 0 && (!W1 || !W3 || !W2)) return MOE_ERR_INVALID_ARG;
    if (n_streamed > 0 && (!W1_host || !W3_host || !W2_host)) return MOE_ERR_INVALID_ARG;
    // the fused row gather addresses token rows with 32-bit byte offsets
    if (static_cast<unsigned long long>(T) * d * 2ull >= (1ull << 32)) return MOE_ERR_UNSUPPORTED_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n_streamed > 0) {
        const int rc = ensure_streaming(c);
        if (rc != MOE_OK) return rc;
    }
    if (c->prof_armed) c->prof_calls++;
    const size_t per = static_cast<size_t>(d) * f;              // elements of one expert matrix
    auto enqueue_copy = [&](int j) -> int {                    // streamed expert j -> slot j % 2
        const int b = j & 1;
        if (c->freed_valid[b]) MOE_HIP_TRY(hipStreamWaitEvent(c->copy_stream, c->freed[b], 0));
        moe_bf16* dst = reinterpret_cast<moe_bf16*>(c->slot[b]);
        const size_t bytes = per * sizeof(moe_bf16);
        MOE_HIP_TRY(hipMemcpyAsync(dst, W1_host + j * per, bytes, hipMemcpyHostToDevice, c->copy_stream));
        MOE_HIP_TRY(hipMemcpyAsync(dst + per, W3_host + j * per, bytes, hipMemcpyHostToDevice, c->copy_stream));
        MOE_HIP_TRY(hipMemcpyAsync(dst + 2 * per, W2_host + j * per, bytes, hipMemcpyHostToDevice, c->copy_stream));
        MOE_HIP_TRY(hipEventRecord(c->ready[b], c->copy_stream));
        return MOE_OK;
    };
    int rc;
    // The first two transfers start at once and run under the routing and the resident experts.
    for (int j = 0; j < n_streamed && j < 2; ++j)
        if ((rc = enqueue_copy(j)) != MOE_OK) return rc;
    rc = run_stage(c, MOE_STAGE_ROUTE, 1, s, [&] {
        return launch_route(x, w_router, bias, T, d, E, k, c->topk_idx, c->topk_w, nullptr, c->logits, s);
    });
    if (rc != MOE_OK) return rc;
    rc = run_stage(c, MOE_STAGE_PERMUTE, permute_launches(R), s, [&] {
        return launch_permute(c->topk_idx, R, E, c->counts, c->offsets, c->perm, c->inv_perm,
                              c->scratch, s);
    });
    if (rc != MOE_OK) return rc;
    // experts [e0, e0 + n) with weights at w1/w3/w2; rows outside those groups are not touched
    auto ffn = [&](int e0, int n, const moe_bf16* w1, const moe_bf16* w3, const moe_bf16* w2) -> int {
        const int hint = static_cast<int>(static_cast<long long>(R) * n / E);
        int r = run_stage(c, MOE_STAGE_GATEUP, 1, s, [&] {
            return launch_gateup(c->gemm, x, c->perm, k, c->offsets + e0, R, hint, d, f, n, w1, w3, c->H, s);
        });
        if (r != MOE_OK) return r;
        return run_stage(c, MOE_STAGE_DOWN, 1, s, [&] {
            return launch_down(c->gemm, c->H, c->offsets + e0, R, hint, d, f, n, w2, expert_out(c), c->y_perm_f32 != nullptr, s);
        });
    };
    if (E_res > 0 && (rc = ffn(0, E_res, W1, W3, W2)) != MOE_OK) return rc;
    for (int j = 0; j < n_streamed; ++j) {
        const int b = j & 1;
        MOE_HIP_TRY(hipStreamWaitEvent(s, c->ready[b], 0));
        const moe_bf16* w = reinterpret_cast<const moe_bf16*>(c->slot[b]);
        if ((rc = ffn(E_res + j, 1, w, w + per, w + 2 * per)) != MOE_OK) return rc;
        MOE_HIP_TRY(hipEventRecord(c->freed[b], s));
        c->freed_valid[b] = true;
        if (j + 2 < n_streamed && (rc = enqueue_copy(j + 2)) != MOE_OK) return rc;
    }
    return run_stage(c, MOE_STAGE_COMBINE, 1, s, [&] {
        return launch_combine(expert_out(c), c->y_perm_f32 != nullptr, c->inv_perm, c->topk_w, T, d, k, y, s);
    });
}

int moe_last_routing(moe_ctx* c, int32_t T, int32_t* topk_idx, float* topk_w, int32_t* counts,
                     int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* stream) {
    if (!c || T < 0 || T > c->shape.T_max) return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t R = static_cast<size_t>(T) * c->shape.k, E = static_cast<size_t>(c->shape.E);
    auto copy = [&](void* dst, const void* src, size_t bytes) -> int {
        if (!dst || bytes == 0) return MOE_OK;
        return hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, s) == hipSuccess ? MOE_OK
                                                                                        : MOE_ERR_HIP;
    };
    int rc = copy(topk_idx, c->topk_idx, R * 4);
    if (rc == MOE_OK) rc = copy(topk_w, c->topk_w, R * 4);
    if (rc == MOE_OK) rc = copy(counts, c->counts, E * 4);
    if (rc == MOE_OK) rc = copy(offsets, c->offsets, (E + 1) * 4);
    if (rc == MOE_OK) rc = copy(perm, c->perm, R * 4);
    if (rc == MOE_OK) rc = copy(inv_perm, c->inv_perm, R * 4);
    return rc;
}

int moe_profile_begin(moe_ctx* c, int32_t max_calls) {
    if (!c || max_calls < 1) return MOE_ERR_INVALID_ARG;
    for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
    c->prof_events.clear();
    c->prof_stage.clear();
    c->prof_call.clear();
    for (auto& v : c->prof_launches) v = 0;
    c->prof_armed = true;
    c->prof_max_calls = max_calls;
    c->prof_calls = 0;
    return MOE_OK;
}

namespace {
// Waits for the recorded intervals and adds every one to its stage's total and, if asked for,
// to its (call, stage) cell; disarms and releases the events.
int profile_collect(moe_ctx* c, double* stage_ms, double* per_call_ms, int32_t capacity_calls,
                    int64_t* stage_launches, int32_t* calls) {
    if (!c || !stage_launches || !calls) return MOE_ERR_INVALID_ARG;
    if (!c->prof_armed) return MOE_ERR_INVALID_ARG;
    c->prof_armed = false;
    const int32_t n_calls = c->prof_calls < c->prof_max_calls ? c->prof_calls : c->prof_max_calls;
    for (int i = 0; i < MOE_NUM_STAGES; ++i) {
        if (stage_ms) stage_ms[i] = 0.0;
        stage_launches[i] = c->prof_launches[i];
    }
    if (per_call_ms)
        for (int64_t i = 0; i < static_cast<int64_t>(capacity_calls) * MOE_NUM_STAGES; ++i) per_call_ms[i] = 0.0;
    int rc = MOE_OK;
    for (size_t i = 0; i < c->prof_stage.size(); ++i) {
        hipEvent_t e0 = c->prof_events[2 * i], e1 = c->prof_events[2 * i + 1];
        float ms = 0.f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
            rc = MOE_ERR_HIP;
            continue;
        }
        if (stage_ms) stage_ms[c->prof_stage[i]] += ms;
        const int call = c->prof_call[i];
        if (per_call_ms && call >= 0 && call < capacity_calls)
            per_call_ms[static_cast<size_t>(call) * MOE_NUM_STAGES + c->prof_stage[i]] += ms;
    }
    *calls = n_calls;
    for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
    c->prof_events.clear();
    c->prof_stage.clear();
    c->prof_call.clear();
    return rc;
}
}  // namespace

int moe_profile_end(moe_ctx* c, double* stage_ms, int64_t* stage_launches, int32_t* calls) {
    if (!stage_ms) return MOE_ERR_INVALID_ARG;
    return profile_collect(c, stage_ms, nullptr, 0, stage_launches, calls);
}

int moe_profile_end_per_call(moe_ctx* c, double* per_call_ms, int32_t capacity_calls,
                             int64_t* stage_launches, int32_t* calls) {
    if (!per_call_ms || capacity_calls < 1) return MOE_ERR_INVALID_ARG;
    return profile_collect(c, nullptr, per_call_ms, capacity_calls, stage_launches, calls);
}

/* Tuning/testing knob of one context: force the expert-GEMM tile configuration (0 large, 1 medium,
 * 2 small, 3 tiny rows-per-expert, 4 the 96-row medium tile), or -1 for the automatic choice; +16 never loads weights as
 * non-temporal, +32 always does (medium and small tiles); +64 makes the layer calls write the
 * gathered rows to the workspace instead of reading them through the permutation; +128 keeps the
 * large tiles of a last, partial round whole; +256 / +512 run the large tiles with eight / four
 * wavefronts. All settings give identical bits. */
int moe_set_gemm_config(moe_ctx* c, int config) {
    if (!c) return MOE_ERR_INVALID_ARG;
    int stream_mode = -1;
    bool materialise = false, split = true;
    int large_waves = 0;
    if (config >= 511) { large_waves = 4; config -= 512; }
    else if (config >= 255) { large_waves = 8; config -= 256; }
    if (config >= 127) { split = false; config -= 128; }
    if (config >= 63) { materialise = true; config -= 64; }
    if (config >= 31) { stream_mode = 1; config -= 32; }
    else if (config >= 15) { stream_mode = 0; config -= 16; }
    if (config < -1 || config > 4) return MOE_ERR_INVALID_ARG;
    c->gemm.materialise_gather = materialise;
    c->gemm.split_last_round = split;
    c->gemm.large_tile_waves = large_waves;
    c->gemm.forced_config = config;
    c->gemm.stream_mode = stream_mode;
    return MOE_OK;
}

int moe_set_expert_output_fp32(moe_ctx* c, int enable) {
    if (!c) return MOE_ERR_INVALID_ARG;
    if (!on_own_device(c)) return MOE_ERR_INVALID_ARG;
    if (enable) {
        if (c->y_perm_f32) return MOE_OK;
        const size_t bytes = static_cast<size_t>(c->shape.T_max) * c->shape.k * c->shape.d_model * sizeof(float);
        void* p = nullptr;
        if (hipMalloc(&p, bytes > 0 ? bytes : 256) != hipSuccess) {
            (void)hipGetLastError();
            return MOE_ERR_WORKSPACE;
        }
        c->y_perm_f32 = static_cast<float*>(p);
        return MOE_OK;
    }
    if (c->y_perm_f32) {
        // the caller has drained the stream (as for moe_destroy)
        const hipError_t err = hipFree(c->y_perm_f32);
        c->y_perm_f32 = nullptr;
        if (err != hipSuccess) return MOE_ERR_HIP;
    }
    return MOE_OK;
}

}  // extern "C"
