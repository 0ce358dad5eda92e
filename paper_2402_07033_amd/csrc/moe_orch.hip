// Execution of a layer whose expert matrices do not all fit in device memory: the paper's
// placement (Sec. 3.4), latency model (Sec. 3.3) and Algorithm 1, over the expert-FFN
// kernels of this library.  Host logic plus one host-side expert kernel (case (c) of
// Sec. 3.2); see include/moe_orch.h.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <new>
#include <numeric>
#include <thread>
#include <vector>

#include "moe_internal.h"
#include "moe_orch.h"

// ------------------------------------------------------------- host logic ----

extern "C" int moe_orch_place(const double* popularity, int L, int E, int capacity,
                              uint8_t* at_gpu) {
    if (!popularity || !at_gpu || L < 1 || E < 1 || capacity < 0) return MOE_ERR_INVALID_ARG;
    const long n = (long)L * E;
    for (long i = 0; i < n; i++)
        if (!(popularity[i] >= 0.0)) return MOE_ERR_INVALID_ARG;  // negative or NaN
    std::vector<long> order(n);
    std::iota(order.begin(), order.end(), 0L);
    // most popular first; the lower index among equals
    std::stable_sort(order.begin(), order.end(),
                     [&](long a, long b) { return popularity[a] > popularity[b]; });
    std::memset(at_gpu, 0, (size_t)n);
    const long take = capacity < n ? capacity : n;
    for (long i = 0; i < take; i++) at_gpu[order[i]] = 1;
    return MOE_OK;
}

extern "C" double moe_orch_hit_rate(const double* popularity, const uint8_t* at_gpu, int L, int E) {
    if (!popularity || !at_gpu || L < 1 || E < 1) return 0.0;
    double hit = 0.0, all = 0.0;
    for (long i = 0; i < (long)L * E; i++) {
        all += popularity[i];
        if (at_gpu[i]) hit += popularity[i];
    }
    return all > 0.0 ? hit / all : 0.0;
}

extern "C" int moe_orch_decide(const uint8_t* at_gpu, const int32_t* inp_size, int E,
                               const moe_orch_latency_t* lat, int32_t* decisions) {
    if (!at_gpu || !inp_size || !lat || !decisions || E < 1) return MOE_ERR_INVALID_ARG;
    for (int j = 0; j < E; j++) {
        const int s = inp_size[j];
        if (s <= 0) {
            decisions[j] = MOE_ORCH_SKIP;
        } else if (at_gpu[j]) {
            decisions[j] = MOE_ORCH_GPU_RESIDENT;
        } else {
            const double cpu_lat = lat->cpu_lat_us_per_row * (double)s;  // grows with the input
            const double gpu_lat = lat->gpu_lat_us;                      // does not
            decisions[j] = (cpu_lat > gpu_lat + lat->transfer_lat_us) ? MOE_ORCH_GPU_TRANSFER
                                                                      : MOE_ORCH_CPU;
        }
    }
    return MOE_OK;
}

// ------------------------------------------------ host-side expert (case c) ----

static int orch_threads() {
    unsigned n = std::thread::hardware_concurrency();
    if (const char* env = std::getenv("OMP_NUM_THREADS")) {
        const int v = std::atoi(env);
        if (v > 0) n = (unsigned)v;
    }
    return (int)(n < 1 ? 1 : (n > 64 ? 64 : n));
}

// fn(t, nt) on nt threads
template <class Fn>
static void orch_parallel(int nt, Fn fn) {
    std::vector<std::thread> th;
    th.reserve((size_t)nt);
    for (int t = 1; t < nt; t++) th.emplace_back([=] { fn(t, nt); });
    fn(0, nt);
    for (auto& x : th) x.join();
}

static inline float orch_bf16(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float v;
    std::memcpy(&v, &u, 4);
    return v;
}

// out[i, c0:c1) = sum_r x[i, r] * W[r, c0:c1) for i < s; W bf16 [K, C] row-major.  Every
// weight row segment is widened once and used for all s rows, so the matrix is read once
// whatever s is.
static void orch_rows_times_matrix(const float* x, int s, int K, const uint16_t* W, int C, int c0,
                                   int c1, float* out /*[s][c1-c0]*/, float* wrow /*[c1-c0]*/) {
    const int cw = c1 - c0;
    std::fill(out, out + (size_t)s * cw, 0.f);
    for (int r = 0; r < K; r++) {
        const uint16_t* w = W + (size_t)r * C + c0;
        for (int c = 0; c < cw; c++) wrow[c] = orch_bf16(w[c]);
        for (int i = 0; i < s; i++) {
            const float xv = x[(size_t)i * K + r];
            float* o = out + (size_t)i * cw;
            for (int c = 0; c < cw; c++) o[c] += xv * wrow[c];
        }
    }
}

extern "C" int moe_orch_cpu_expert_ffn(const float* x, int s, const uint16_t* w1,
                                       const uint16_t* w3, const uint16_t* w2, int d, int f,
                                       float* y) {
    if (s < 0 || d < 1 || f < 1) return MOE_ERR_INVALID_ARG;
    if (s == 0) return MOE_OK;
    if (!x || !w1 || !w3 || !w2 || !y) return MOE_ERR_INVALID_ARG;
    std::vector<float> h((size_t)s * f);
    const int nt = orch_threads();
    // first projection and SiLU * mul: threads own column ranges of f
    orch_parallel(nt, [&](int t, int n) {
        const int c0 = (int)((long)f * t / n), c1 = (int)((long)f * (t + 1) / n), cw = c1 - c0;
        if (cw <= 0) return;
        std::vector<float> a((size_t)s * cw), b((size_t)s * cw), wrow((size_t)cw);
        orch_rows_times_matrix(x, s, d, w1, f, c0, c1, a.data(), wrow.data());
        orch_rows_times_matrix(x, s, d, w3, f, c0, c1, b.data(), wrow.data());
        for (int i = 0; i < s; i++)
            for (int c = 0; c < cw; c++) {
                const float av = a[(size_t)i * cw + c];
                h[(size_t)i * f + c0 + c] = av / (1.0f + std::exp(-av)) * b[(size_t)i * cw + c];
            }
    });
    // second projection: threads own column ranges of d
    orch_parallel(nt, [&](int t, int n) {
        const int q0 = (int)((long)d * t / n), q1 = (int)((long)d * (t + 1) / n), qw = q1 - q0;
        if (qw <= 0) return;
        std::vector<float> o((size_t)s * qw), wrow((size_t)qw);
        orch_rows_times_matrix(h.data(), s, f, w2, d, q0, q1, o.data(), wrow.data());
        for (int i = 0; i < s; i++)
            std::memcpy(y + (size_t)i * d + q0, o.data() + (size_t)i * qw, sizeof(float) * (size_t)qw);
    });
    return MOE_OK;
}

// ------------------------------------------------------------ split layer ----

struct moe_orch_layer {
    int E, d, f, max_rows, device;
    std::vector<uint8_t> at_gpu;
    std::vector<moe_weights*> resident;      // per expert: single-expert packed handle, or null
    std::vector<uint16_t*> h_w1, h_w3, h_w2;  // per expert: pinned raw matrices, or null
    // staging slot of case (b): raw device copies and the packed single-expert handle
    uint16_t *s_w1 = nullptr, *s_w3 = nullptr, *s_w2 = nullptr;
    moe_weights* stage = nullptr;
    int32_t* d_off2 = nullptr;   // device [E][2]: (0, s_j) of every expert run on the device
    int32_t* h_off = nullptr;    // pinned [E+1]: offsets as copied back
    int32_t* h_off2 = nullptr;   // pinned [E][2]
    float *h_x = nullptr, *h_y = nullptr;  // pinned [max_rows, d]: rows and results of case (c)
    hipEvent_t ev = nullptr;
};

static void orch_destroy(moe_orch_layer* Lr) {
    if (!Lr) return;
    for (auto* w : Lr->resident)
        if (w) (void)moe_weights_free_impl(w);
    for (auto* p : Lr->h_w1) if (p) (void)hipHostFree(p);
    for (auto* p : Lr->h_w3) if (p) (void)hipHostFree(p);
    for (auto* p : Lr->h_w2) if (p) (void)hipHostFree(p);
    if (Lr->stage) (void)moe_weights_free_impl(Lr->stage);
    void* dev[4] = {Lr->s_w1, Lr->s_w3, Lr->s_w2, Lr->d_off2};
    for (void* p : dev) if (p) (void)hipFree(p);
    void* host[5] = {Lr->h_off, Lr->h_off2, Lr->h_x, Lr->h_y, nullptr};
    for (void* p : host) if (p) (void)hipHostFree(p);
    if (Lr->ev) (void)hipEventDestroy(Lr->ev);
    (void)hipGetLastError();
    delete Lr;
}

extern "C" int moe_orch_layer_free(moe_orch_layer_t* layer) {
    if (!layer) return MOE_OK;
    if (hipDeviceSynchronize() != hipSuccess) (void)hipGetLastError();
    orch_destroy(layer);
    return MOE_OK;
}

#define ORCH_TRY(expr)                  \
    do {                                \
        if ((expr) != hipSuccess) {     \
            (void)hipGetLastError();    \
            orch_destroy(Lr);           \
            return MOE_ERR_HIP;         \
        }                               \
    } while (0)

extern "C" int moe_orch_layer_create(const uint16_t* w1, const uint16_t* w3, const uint16_t* w2,
                                     int E, int d, int f, const uint8_t* at_gpu, int max_rows,
                                     moe_orch_layer_t** out, void* stream) {
    if (!out) return MOE_ERR_INVALID_ARG;
    *out = nullptr;
    if (!w1 || !w3 || !w2 || !at_gpu || E < 1 || E > MOE_MAX_E || d < 64 || d % 64 || f < 64 ||
        f % 64 || max_rows < 1 || max_rows >= MOE_MAX_N)
        return MOE_ERR_INVALID_ARG;
    moe_orch_layer* Lr = new (std::nothrow) moe_orch_layer();
    if (!Lr) return MOE_ERR_HIP;
    Lr->E = E; Lr->d = d; Lr->f = f; Lr->max_rows = max_rows;
    Lr->device = moe_current_device();
    Lr->at_gpu.assign(at_gpu, at_gpu + E);
    Lr->resident.assign((size_t)E, nullptr);
    Lr->h_w1.assign((size_t)E, nullptr);
    Lr->h_w3.assign((size_t)E, nullptr);
    Lr->h_w2.assign((size_t)E, nullptr);
    hipStream_t s = (hipStream_t)stream;
    const size_t mat = (size_t)d * f, mat_bytes = mat * sizeof(uint16_t);
    ORCH_TRY(hipMalloc((void**)&Lr->s_w1, mat_bytes));
    ORCH_TRY(hipMalloc((void**)&Lr->s_w3, mat_bytes));
    ORCH_TRY(hipMalloc((void**)&Lr->s_w2, mat_bytes));
    ORCH_TRY(hipMalloc((void**)&Lr->d_off2, sizeof(int32_t) * 2 * (size_t)E));
    ORCH_TRY(hipHostMalloc((void**)&Lr->h_off, sizeof(int32_t) * (size_t)(E + 1), hipHostMallocDefault));
    ORCH_TRY(hipHostMalloc((void**)&Lr->h_off2, sizeof(int32_t) * 2 * (size_t)E, hipHostMallocDefault));
    ORCH_TRY(hipHostMalloc((void**)&Lr->h_x, sizeof(float) * (size_t)max_rows * d, hipHostMallocDefault));
    ORCH_TRY(hipHostMalloc((void**)&Lr->h_y, sizeof(float) * (size_t)max_rows * d, hipHostMallocDefault));
    ORCH_TRY(hipEventCreateWithFlags(&Lr->ev, hipEventDisableTiming));
    for (int e = 0; e < E; e++) {
        const uint16_t *a = w1 + (size_t)e * mat, *b = w3 + (size_t)e * mat, *c = w2 + (size_t)e * mat;
        if (at_gpu[e]) {
            // through the staging buffers: upload, then pack into the expert's own handle
            ORCH_TRY(hipMemcpyAsync(Lr->s_w1, a, mat_bytes, hipMemcpyHostToDevice, s));
            ORCH_TRY(hipMemcpyAsync(Lr->s_w3, b, mat_bytes, hipMemcpyHostToDevice, s));
            ORCH_TRY(hipMemcpyAsync(Lr->s_w2, c, mat_bytes, hipMemcpyHostToDevice, s));
            if (moe_weights_pack_impl(Lr->s_w1, Lr->s_w3, Lr->s_w2, 1, d, f, MOE_BF16,
                                      &Lr->resident[(size_t)e], s) != MOE_OK) {
                orch_destroy(Lr);
                return MOE_ERR_HIP;
            }
            // the caller's arrays are pageable: the copies above have completed on return, but
            // the pack kernels still read the staging buffers
            ORCH_TRY(hipStreamSynchronize(s));
        } else {
            ORCH_TRY(hipHostMalloc((void**)&Lr->h_w1[(size_t)e], mat_bytes, hipHostMallocDefault));
            ORCH_TRY(hipHostMalloc((void**)&Lr->h_w3[(size_t)e], mat_bytes, hipHostMallocDefault));
            ORCH_TRY(hipHostMalloc((void**)&Lr->h_w2[(size_t)e], mat_bytes, hipHostMallocDefault));
            std::memcpy(Lr->h_w1[(size_t)e], a, mat_bytes);
            std::memcpy(Lr->h_w3[(size_t)e], b, mat_bytes);
            std::memcpy(Lr->h_w2[(size_t)e], c, mat_bytes);
        }
    }
    // the staging handle: packed buffers of one expert, filled by every case (b)
    ORCH_TRY(hipMemsetAsync(Lr->s_w1, 0, mat_bytes, s));
    ORCH_TRY(hipMemsetAsync(Lr->s_w3, 0, mat_bytes, s));
    ORCH_TRY(hipMemsetAsync(Lr->s_w2, 0, mat_bytes, s));
    if (moe_weights_pack_impl(Lr->s_w1, Lr->s_w3, Lr->s_w2, 1, d, f, MOE_BF16, &Lr->stage, s) != MOE_OK) {
        orch_destroy(Lr);
        return MOE_ERR_HIP;
    }
    ORCH_TRY(hipStreamSynchronize(s));
    *out = Lr;
    return MOE_OK;
}
#undef ORCH_TRY

// Case (b): weights of expert e into the staging slot (pinned host -> device, then repack).
static int orch_stage_expert(moe_orch_layer* Lr, int e, hipStream_t s) {
    const size_t mat_bytes = (size_t)Lr->d * Lr->f * sizeof(uint16_t);
    MOE_HIP_TRY(hipMemcpyAsync(Lr->s_w1, Lr->h_w1[(size_t)e], mat_bytes, hipMemcpyHostToDevice, s));
    MOE_HIP_TRY(hipMemcpyAsync(Lr->s_w3, Lr->h_w3[(size_t)e], mat_bytes, hipMemcpyHostToDevice, s));
    MOE_HIP_TRY(hipMemcpyAsync(Lr->s_w2, Lr->h_w2[(size_t)e], mat_bytes, hipMemcpyHostToDevice, s));
    return moe_weights_repack_impl(Lr->stage, Lr->s_w1, Lr->s_w3, Lr->s_w2, s);
}

static int orch_check_call(const moe_orch_layer* Lr, int N, const void* ws, size_t ws_bytes) {
    if (!Lr || N < 0 || N > Lr->max_rows) return MOE_ERR_INVALID_ARG;
    if (!ws || (((uintptr_t)ws) & 255u)) return MOE_ERR_WORKSPACE;
    if (ws_bytes < moe_expert_ffn_workspace(N > 0 ? N : 1, 1, Lr->d, Lr->f, MOE_F32)) return MOE_ERR_WORKSPACE;
    return MOE_OK;
}

extern "C" int moe_orch_expert_ffn(moe_orch_layer_t* Lr, const moe_orch_latency_t* lat,
                                   const float* xg, const int32_t* offsets, int N, void* workspace,
                                   size_t workspace_bytes, float* yg, int32_t* decisions,
                                   void* stream) {
    int rc = orch_check_call(Lr, N, workspace, workspace_bytes);
    if (rc != MOE_OK) return rc;
    if (!lat || !offsets) return MOE_ERR_INVALID_ARG;
    if (N == 0) {
        if (decisions) for (int j = 0; j < Lr->E; j++) decisions[j] = MOE_ORCH_SKIP;
        return MOE_OK;
    }
    if (!xg || !yg || !moe_aligned16(xg) || !moe_aligned16(yg)) return MOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int E = Lr->E, d = Lr->d;
    // The decision is the host's (Sec. 3.3 "Execution"): the per-expert input sizes come back
    // first.  This wait also covers the previous call's copies out of h_y.
    MOE_HIP_TRY(hipMemcpyAsync(Lr->h_off, offsets, sizeof(int32_t) * (size_t)(E + 1),
                               hipMemcpyDeviceToHost, s));
    MOE_HIP_TRY(hipStreamSynchronize(s));
    std::vector<int32_t> size((size_t)E), dec((size_t)E);
    for (int j = 0; j < E; j++) {
        int lo = Lr->h_off[j], hi = Lr->h_off[j + 1];
        lo = lo < 0 ? 0 : (lo > N ? N : lo);
        hi = hi < lo ? lo : (hi > N ? N : hi);
        Lr->h_off[j] = lo;
        size[(size_t)j] = hi - lo;
        Lr->h_off2[2 * j] = 0;
        Lr->h_off2[2 * j + 1] = hi - lo;
    }
    rc = moe_orch_decide(Lr->at_gpu.data(), size.data(), E, lat, dec.data());
    if (rc != MOE_OK) return rc;
    if (decisions) std::memcpy(decisions, dec.data(), sizeof(int32_t) * (size_t)E);

    // case (c) first: its rows travel to the host while the device runs the other experts
    bool any_cpu = false;
    for (int j = 0; j < E; j++)
        if (dec[(size_t)j] == MOE_ORCH_CPU) {
            any_cpu = true;
            MOE_HIP_TRY(hipMemcpyAsync(Lr->h_x + (size_t)Lr->h_off[j] * d, xg + (size_t)Lr->h_off[j] * d,
                                       sizeof(float) * (size_t)size[(size_t)j] * d, hipMemcpyDeviceToHost, s));
        }
    if (any_cpu) MOE_HIP_TRY(hipEventRecord(Lr->ev, s));
    MOE_HIP_TRY(hipMemcpyAsync(Lr->d_off2, Lr->h_off2, sizeof(int32_t) * 2 * (size_t)E,
                               hipMemcpyHostToDevice, s));
    // cases (a) and (b): one expert per call, as Algorithm 1 walks them
    for (int pass = 0; pass < 2; pass++)
        for (int j = 0; j < E; j++) {
            const int want = pass == 0 ? MOE_ORCH_GPU_RESIDENT : MOE_ORCH_GPU_TRANSFER;
            if (dec[(size_t)j] != want) continue;
            const moe_weights* Wj = Lr->resident[(size_t)j];
            if (pass == 1) {
                rc = orch_stage_expert(Lr, j, s);
                if (rc != MOE_OK) return rc;
                Wj = Lr->stage;
            }
            const size_t row0 = (size_t)Lr->h_off[j];
            rc = moe_expert_ffn(Wj, xg + row0 * d, MOE_F32, Lr->d_off2 + 2 * j, size[(size_t)j],
                                workspace, workspace_bytes, yg + row0 * d, s);
            if (rc != MOE_OK) return rc;
        }
    if (any_cpu) {
        MOE_HIP_TRY(hipEventSynchronize(Lr->ev));
        for (int j = 0; j < E; j++) {
            if (dec[(size_t)j] != MOE_ORCH_CPU) continue;
            const size_t row0 = (size_t)Lr->h_off[j];
            rc = moe_orch_cpu_expert_ffn(Lr->h_x + row0 * d, size[(size_t)j], Lr->h_w1[(size_t)j],
                                         Lr->h_w3[(size_t)j], Lr->h_w2[(size_t)j], d, Lr->f,
                                         Lr->h_y + row0 * d);
            if (rc != MOE_OK) return rc;
            MOE_HIP_TRY(hipMemcpyAsync(yg + row0 * d, Lr->h_y + row0 * d,
                                       sizeof(float) * (size_t)size[(size_t)j] * d, hipMemcpyHostToDevice, s));
        }
    }
    return MOE_OK;
}

extern "C" int moe_orch_calibrate(moe_orch_layer_t* Lr, void* workspace, size_t workspace_bytes,
                                  moe_orch_latency_t* lat, void* stream) {
    int rc = orch_check_call(Lr, Lr ? (Lr->max_rows < 16 ? Lr->max_rows : 16) : 0, workspace,
                             workspace_bytes);
    if (rc != MOE_OK) return rc;
    if (!lat) return MOE_ERR_INVALID_ARG;
    int e_host = -1;
    for (int j = 0; j < Lr->E; j++)
        if (!Lr->at_gpu[(size_t)j]) { e_host = j; break; }
    if (e_host < 0) return MOE_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    const int d = Lr->d;
    const int rows = Lr->max_rows < 16 ? Lr->max_rows : 16;
    // probe rows: a fixed pattern in the pinned buffer; the device runs read a device copy
    // that lives for the duration of this call (initialisation, so allocating is fine)
    float *dx = nullptr, *dy = nullptr;
    MOE_HIP_TRY(hipMalloc((void**)&dx, sizeof(float) * (size_t)rows * d));
    if (hipMalloc((void**)&dy, sizeof(float) * (size_t)rows * d) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(dx);
        return MOE_ERR_HIP;
    }
    for (size_t i = 0; i < (size_t)rows * d; i++) Lr->h_x[i] = 0.25f * (float)((int)(i % 13) - 6);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    auto cleanup = [&](int code) {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
        (void)hipFree(dx);
        (void)hipFree(dy);
        (void)hipGetLastError();
        return code;
    };
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return cleanup(MOE_ERR_HIP);
    if (hipMemcpyAsync(dx, Lr->h_x, sizeof(float) * (size_t)rows * d, hipMemcpyHostToDevice, s) != hipSuccess)
        return cleanup(MOE_ERR_HIP);
    auto elapsed_us = [&](double& us) -> bool {
        float ms = 0.f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return false;
        us = (double)ms * 1e3;
        return true;
    };
    // transfer_lat: one expert's matrices into the staging slot, repacked (twice; the second)
    double t_transfer = 0.0;
    for (int rep = 0; rep < 2; rep++) {
        if (hipEventRecord(e0, s) != hipSuccess) return cleanup(MOE_ERR_HIP);
        if (orch_stage_expert(Lr, e_host, s) != MOE_OK) return cleanup(MOE_ERR_HIP);
        if (hipEventRecord(e1, s) != hipSuccess || !elapsed_us(t_transfer)) return cleanup(MOE_ERR_HIP);
    }
    // gpu_lat: the staged expert at 1 and `rows` rows (warm-up first), mean of the two
    double t_gpu = 0.0;
    const int sizes_gpu[2] = {1, rows};
    for (int i = 0; i < 2; i++) {
        Lr->h_off2[0] = 0;
        Lr->h_off2[1] = sizes_gpu[i];
        if (hipMemcpyAsync(Lr->d_off2, Lr->h_off2, sizeof(int32_t) * 2, hipMemcpyHostToDevice, s) != hipSuccess)
            return cleanup(MOE_ERR_HIP);
        double us = 0.0;
        for (int rep = 0; rep < 3; rep++) {
            if (hipEventRecord(e0, s) != hipSuccess) return cleanup(MOE_ERR_HIP);
            if (moe_expert_ffn(Lr->stage, dx, MOE_F32, Lr->d_off2, sizes_gpu[i], workspace,
                               workspace_bytes, dy, s) != MOE_OK)
                return cleanup(MOE_ERR_HIP);
            if (hipEventRecord(e1, s) != hipSuccess || !elapsed_us(us)) return cleanup(MOE_ERR_HIP);
        }
        t_gpu += us / 2.0;
    }
    // cpu_lat: the host kernel at 1, 2, 4 rows; slope of the least-squares line through 0
    double sxy = 0.0, sxx = 0.0;
    for (int sz : {1, 2, 4}) {
        if (sz > rows) break;
        const auto c0 = std::chrono::steady_clock::now();
        if (moe_orch_cpu_expert_ffn(Lr->h_x, sz, Lr->h_w1[(size_t)e_host], Lr->h_w3[(size_t)e_host],
                                    Lr->h_w2[(size_t)e_host], d, Lr->f, Lr->h_y) != MOE_OK)
            return cleanup(MOE_ERR_HIP);
        const double us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - c0).count();
        sxy += us * sz;
        sxx += (double)sz * sz;
    }
    lat->gpu_lat_us = t_gpu;
    lat->cpu_lat_us_per_row = sxx > 0.0 ? sxy / sxx : 0.0;
    lat->transfer_lat_us = t_transfer;
    if (hipStreamSynchronize(s) != hipSuccess) return cleanup(MOE_ERR_HIP);
    return cleanup(MOE_OK);
}
