// libdbsn host side: the C ABI declared in include/dbsn.h.  Argument checks, arena layout,
// kernel launches.  No device memory is allocated here.
#include "dbsn.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "dbsn_deform_kernels.h"
#include "dbsn_mlp_kernels.h"

using namespace dbsn;

namespace {

thread_local std::string g_err;

int32_t fail(int32_t code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(DBSN_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

constexpr size_t kAlign = 256;
size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }
constexpr int kArenaGroups = 512;  // partial-sum rows the arena is sized for (>= workgroups launched)

bool shape_ok(const int32_t* sizes, int32_t n_sizes) {
    if (!sizes || n_sizes < 2 || n_sizes > DBSN_MAX_LAYERS + 1) return false;
    for (int i = 0; i < n_sizes; ++i)
        if (sizes[i] < 1 || sizes[i] > DBSN_MAX_WIDTH) return false;
    return sizes[n_sizes - 1] <= DBSN_MAX_CLASSES;
}

struct ArenaPlan {
    size_t W[kMaxLayers + 1], b[kMaxLayers + 1], x[kMaxLayers + 1], d[kMaxLayers + 1];
    size_t gpart[2], flags, total;
    int ld[kMaxLayers + 1], gld;
};

ArenaPlan plan_arena(const int32_t* sizes, int32_t n_sizes) {
    ArenaPlan p{};
    size_t off = 0;
    int maxw = 0;
    for (int l = 1; l < n_sizes; ++l) {
        const int nin = sizes[l - 1], nout = sizes[l];
        p.ld[l] = (nin + 3) / 4 * 4;
        p.W[l] = off; off = align_up(off + sizeof(float) * (size_t)nout * p.ld[l]);
        p.b[l] = off; off = align_up(off + sizeof(float) * (size_t)nout);
        p.x[l] = off; off = align_up(off + sizeof(float) * (size_t)nout);
        p.d[l] = off; off = align_up(off + sizeof(float) * (size_t)nout);
        if (nin > maxw) maxw = nin;
    }
    p.gld = (maxw + 63) / 64 * 64;
    for (int k = 0; k < 2; ++k) {
        p.gpart[k] = off;
        off = align_up(off + sizeof(float) * (size_t)kArenaGroups * p.gld);
    }
    p.flags = off; off = align_up(off + 256);
    p.total = off;
    return p;
}

}  // namespace

struct dbsn_mlp {
    Net net{};
    std::vector<int32_t> sizes;
    ArenaPlan plan{};
    char* arena = nullptr;
    hipStream_t stream = nullptr;
    int mode = DBSN_MODE_PERSISTENT;
    int maxnch = 0;
    unsigned bar_base = 0;
    int device = 0;
    size_t lds_limit = 0;
    bool persistent_ready = false;
};

namespace {

template <int NCH>
int32_t launch_fwd(dbsn_mlp* m, int l, const float* x0) {
    const size_t lds = sizeof(float) * (size_t)(NCH * 256);
    hipLaunchKernelGGL(k_fwd<NCH>, dim3(m->net.G), dim3(kThreads), lds, m->stream, m->net, l, x0);
    return DBSN_OK;
}
template <int NCH>
int32_t launch_bwd(dbsn_mlp* m, int l, const float* x0, float eta) {
    const size_t lds = sizeof(float) * (size_t)phase_lds_floats(NCH);
    if (lds > 64 * 1024)
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_bwd<NCH>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(k_bwd<NCH>, dim3(m->net.G), dim3(kThreads), lds, m->stream, m->net, l, x0, eta);
    return DBSN_OK;
}

int32_t fwd_layer(dbsn_mlp* m, int l, const float* x0) {
    int32_t rc = DBSN_E_SHAPE;
    DBSN_NCH_SWITCH(16, m->net.lay[l].nch, rc = launch_fwd<N>(m, l, x0));
    return rc;
}
int32_t bwd_layer(dbsn_mlp* m, int l, const float* x0, float eta) {
    int32_t rc = DBSN_E_SHAPE;
    DBSN_NCH_SWITCH(16, m->net.lay[l].nch, rc = launch_bwd<N>(m, l, x0, eta));
    return rc;
}
int32_t top_layer(dbsn_mlp* m, const float* x0, const int* label_ptr, int label_val, float eta, int train,
                  float* loss_out, int* label_out) {
    const size_t lds = sizeof(float) * (size_t)(m->net.lay[m->net.L].ld + 4 + 2 * kMaxClasses);
    hipLaunchKernelGGL(k_top, dim3(1), dim3(kThreads), lds, m->stream, m->net, x0, label_ptr, label_val, eta,
                       train, loss_out, label_out);
    return DBSN_OK;
}

// forward phases of one sample + output layer (train = 0: no deltas, no update)
int32_t forward_launches(dbsn_mlp* m, const float* x0, int* label_out) {
    for (int l = 1; l < m->net.L; ++l) {
        int32_t rc = fwd_layer(m, l, x0);
        if (rc) return fail(rc, "unsupported layer width");
    }
    return top_layer(m, x0, nullptr, 0, 0.0f, 0, nullptr, label_out);
}

int32_t steps_launches(dbsn_mlp* m, const float* samples, const int* labels, int label_val, int64_t n, float eta,
                       float* loss) {
    const int L = m->net.L, n0 = m->sizes[0];
    for (int64_t s = 0; s < n; ++s) {
        const float* x0 = samples + s * n0;
        for (int l = 1; l < L; ++l) {
            int32_t rc = fwd_layer(m, l, x0);
            if (rc) return fail(rc, "unsupported layer width");
        }
        top_layer(m, x0, labels ? labels + s : nullptr, label_val, eta, 1, loss ? loss + s : nullptr, nullptr);
        for (int l = L - 1; l >= 1; --l) {
            int32_t rc = bwd_layer(m, l, x0, eta);
            if (rc) return rc;
        }
    }
    HIP_TRY(hipGetLastError());
    return DBSN_OK;
}

template <int MAXNCH>
int32_t launch_persistent(dbsn_mlp* m, const float* samples, const int* labels, int label_val, int64_t n,
                          float eta, float* loss) {
    const size_t lds = sizeof(float) * (size_t)phase_lds_floats(MAXNCH);
    const void* fn = reinterpret_cast<const void*>(&k_bp_persistent<MAXNCH>);
    if (lds > m->lds_limit) return fail(DBSN_E_SHAPE, "layer too wide for this device's LDS (%zu B needed)", lds);
    if (!m->persistent_ready) {
        if (lds > 64 * 1024) HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        int per_cu = 0;
        HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kThreads, lds));
        if (per_cu < 1) return fail(DBSN_E_SHAPE, "persistent kernel does not fit on a compute unit");
        m->persistent_ready = true;
    }
    Net net = m->net;
    long long nn = n;
    unsigned base = m->bar_base;
    void* args[] = {&net, &samples, &labels, &label_val, &nn, &eta, &loss, &base};
    HIP_TRY(hipLaunchCooperativeKernel(fn, dim3(net.G), dim3(kThreads), args, (unsigned)lds, m->stream));
    // barriers passed by every workgroup in this launch
    const int L = net.L;
    const unsigned per_step = (L >= 2) ? (unsigned)((L - 1) + (L >= 3 ? L - 2 : 1)) : 0u;
    m->bar_base = base + (unsigned)net.G * per_step * (unsigned)n;
    return DBSN_OK;
}

int32_t steps_persistent(dbsn_mlp* m, const float* samples, const int* labels, int label_val, int64_t n, float eta,
                         float* loss) {
    // keep the barrier counter far from wrapping inside one launch
    const int64_t chunk = 1 << 16;
    for (int64_t a = 0; a < n; a += chunk) {
        const int64_t c = (n - a < chunk) ? n - a : chunk;
        const float* sp = samples + a * m->sizes[0];
        const int* lp = labels ? labels + a : nullptr;
        float* ls = loss ? loss + a : nullptr;
        int32_t rc;
        if (m->maxnch <= 4) rc = launch_persistent<4>(m, sp, lp, label_val, c, eta, ls);
        else if (m->maxnch <= 8) rc = launch_persistent<8>(m, sp, lp, label_val, c, eta, ls);
        else if (m->maxnch <= 10) rc = launch_persistent<10>(m, sp, lp, label_val, c, eta, ls);
        else if (m->maxnch <= 12) rc = launch_persistent<12>(m, sp, lp, label_val, c, eta, ls);
        else rc = launch_persistent<16>(m, sp, lp, label_val, c, eta, ls);
        if (rc) return rc;
    }
    return DBSN_OK;
}

int32_t check_mlp(dbsn_mlp* m) { return m ? DBSN_OK : fail(DBSN_E_ARG, "null network handle"); }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace

extern "C" {

const char* dbsn_last_error(void) { return g_err.c_str(); }

size_t dbsn_mlp_arena_bytes(const int32_t* sizes, int32_t n_sizes) {
    if (!shape_ok(sizes, n_sizes)) return 0;
    return plan_arena(sizes, n_sizes).total;
}

int32_t dbsn_mlp_init(dbsn_mlp** out, const int32_t* sizes, int32_t n_sizes, uint64_t seed, void* arena_dev,
                      size_t arena_bytes, void* hip_stream) {
    if (!out) return fail(DBSN_E_ARG, "out is null");
    *out = nullptr;
    if (!shape_ok(sizes, n_sizes)) return fail(DBSN_E_SHAPE, "unsupported layer sizes");
    if (!arena_dev) return fail(DBSN_E_ARG, "arena is null");
    if (!aligned(arena_dev, kAlign)) return fail(DBSN_E_SHAPE, "arena must be 256-byte aligned");
    ArenaPlan plan = plan_arena(sizes, n_sizes);
    if (arena_bytes < plan.total)
        return fail(DBSN_E_SHAPE, "arena too small: %zu bytes given, %zu needed", arena_bytes, plan.total);

    dbsn_mlp* m = new (std::nothrow) dbsn_mlp();
    if (!m) return fail(DBSN_E_ARG, "out of host memory");
    m->sizes.assign(sizes, sizes + n_sizes);
    m->plan = plan;
    m->arena = static_cast<char*>(arena_dev);
    m->stream = static_cast<hipStream_t>(hip_stream);

    hipError_t e = hipGetDevice(&m->device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, m->device);
    if (e != hipSuccess) {
        delete m;
        return fail(DBSN_E_HIP, "no usable HIP device: %s", hipGetErrorString(e));
    }
    m->lds_limit = prop.sharedMemPerBlock;
    int G = prop.multiProcessorCount;  // one workgroup per compute unit
    if (G > kArenaGroups) G = kArenaGroups;
    int maxw = 0;
    for (int i = 0; i < n_sizes; ++i) maxw = sizes[i] > maxw ? sizes[i] : maxw;
    if ((maxw + G - 1) / G + 1 > kMaxRowsPerGroup) {
        delete m;
        return fail(DBSN_E_SHAPE, "device has too few compute units for this width");
    }
    Net& net = m->net;
    net.L = n_sizes - 1;
    net.G = G;
    net.gld = plan.gld;
    net.spin_limit = 1u << 24;
    for (int l = 1; l <= net.L; ++l) {
        Layer& Ly = net.lay[l];
        Ly.W = reinterpret_cast<float*>(m->arena + plan.W[l]);
        Ly.b = reinterpret_cast<float*>(m->arena + plan.b[l]);
        Ly.x = reinterpret_cast<float*>(m->arena + plan.x[l]);
        Ly.d = reinterpret_cast<float*>(m->arena + plan.d[l]);
        Ly.n_in = sizes[l - 1];
        Ly.n_out = sizes[l];
        Ly.ld = plan.ld[l];
        Ly.nch = nch_for(Ly.ld);
        if (l < net.L && Ly.nch > m->maxnch) m->maxnch = Ly.nch;
    }
    // the output layer's input vector is staged whole in the phase buffer as well
    if (net.L >= 1 && nch_for(net.lay[net.L].ld) > m->maxnch) m->maxnch = nch_for(net.lay[net.L].ld);
    net.gpart[0] = reinterpret_cast<float*>(m->arena + plan.gpart[0]);
    net.gpart[1] = reinterpret_cast<float*>(m->arena + plan.gpart[1]);
    net.bar = reinterpret_cast<unsigned*>(m->arena + plan.flags);
    net.err = reinterpret_cast<int*>(m->arena + plan.flags + 64);

    // everything that is not a weight starts at zero
    e = hipMemsetAsync(m->arena, 0, plan.total, m->stream);
    if (e != hipSuccess) {
        delete m;
        return fail(DBSN_E_HIP, "hipMemsetAsync: %s", hipGetErrorString(e));
    }
    for (int l = 1; l <= net.L; ++l) {
        const long long total = (long long)net.lay[l].n_out * (net.lay[l].ld + 1);
        int blocks = (int)((total + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_init_layer, dim3(blocks), dim3(256), 0, m->stream, net.lay[l],
                           rng_key(seed, (uint64_t)l));
    }
    e = hipGetLastError();
    if (e != hipSuccess) {
        delete m;
        return fail(DBSN_E_HIP, "init launch: %s", hipGetErrorString(e));
    }
    *out = m;
    return DBSN_OK;
}

int32_t dbsn_mlp_free(dbsn_mlp* m) {
    if (!m) return DBSN_OK;
    (void)hipStreamSynchronize(m->stream);
    delete m;
    return DBSN_OK;
}

int32_t dbsn_mlp_set_mode(dbsn_mlp* m, int32_t mode) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (mode != DBSN_MODE_LAUNCHES && mode != DBSN_MODE_PERSISTENT) return fail(DBSN_E_ARG, "unknown mode %d", mode);
    m->mode = mode;
    return DBSN_OK;
}

int32_t dbsn_mlp_set_spin_limit(dbsn_mlp* m, uint32_t polls) {
    if (check_mlp(m)) return DBSN_E_ARG;
    m->net.spin_limit = polls;
    return DBSN_OK;
}

int32_t dbsn_mlp_status(dbsn_mlp* m) {
    if (check_mlp(m)) return DBSN_E_ARG;
    HIP_TRY(hipStreamSynchronize(m->stream));
    int err = 0;
    HIP_TRY(hipMemcpy(&err, m->net.err, sizeof err, hipMemcpyDeviceToHost));
    if (err) {
        // leave the barrier in a clean state for the next launch
        HIP_TRY(hipMemset(m->net.bar, 0, 128));
        m->bar_base = 0;
        return fail(DBSN_E_TIMEOUT, "a grid barrier gave up waiting; weights are undefined");
    }
    return DBSN_OK;
}

int32_t dbsn_mlp_set_weights(dbsn_mlp* m, int32_t layer, const float* W_host, const float* b_host) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (layer < 1 || layer > m->net.L) return fail(DBSN_E_ARG, "layer %d out of range 1..%d", layer, m->net.L);
    const Layer& Ly = m->net.lay[layer];
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (W_host)
        HIP_TRY(hipMemcpy2D(Ly.W, sizeof(float) * Ly.ld, W_host, sizeof(float) * Ly.n_in, sizeof(float) * Ly.n_in,
                            Ly.n_out, hipMemcpyHostToDevice));
    if (b_host) HIP_TRY(hipMemcpy(Ly.b, b_host, sizeof(float) * Ly.n_out, hipMemcpyHostToDevice));
    return DBSN_OK;
}

int32_t dbsn_mlp_get_weights(dbsn_mlp* m, int32_t layer, float* W_host, float* b_host) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (layer < 1 || layer > m->net.L) return fail(DBSN_E_ARG, "layer %d out of range 1..%d", layer, m->net.L);
    const Layer& Ly = m->net.lay[layer];
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (W_host)
        HIP_TRY(hipMemcpy2D(W_host, sizeof(float) * Ly.n_in, Ly.W, sizeof(float) * Ly.ld, sizeof(float) * Ly.n_in,
                            Ly.n_out, hipMemcpyDeviceToHost));
    if (b_host) HIP_TRY(hipMemcpy(b_host, Ly.b, sizeof(float) * Ly.n_out, hipMemcpyDeviceToHost));
    return DBSN_OK;
}

int32_t dbsn_mlp_get_activations(dbsn_mlp* m, int32_t layer, float* x_host) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (layer < 1 || layer > m->net.L) return fail(DBSN_E_ARG, "layer %d out of range 1..%d", layer, m->net.L);
    if (!x_host) return fail(DBSN_E_ARG, "x_host is null");
    HIP_TRY(hipStreamSynchronize(m->stream));
    HIP_TRY(hipMemcpy(x_host, m->net.lay[layer].x, sizeof(float) * m->net.lay[layer].n_out, hipMemcpyDeviceToHost));
    return DBSN_OK;
}

int32_t dbsn_mlp_get_deltas(dbsn_mlp* m, int32_t layer, float* d_host) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (layer < 1 || layer > m->net.L) return fail(DBSN_E_ARG, "layer %d out of range 1..%d", layer, m->net.L);
    if (!d_host) return fail(DBSN_E_ARG, "d_host is null");
    HIP_TRY(hipStreamSynchronize(m->stream));
    HIP_TRY(hipMemcpy(d_host, m->net.lay[layer].d, sizeof(float) * m->net.lay[layer].n_out, hipMemcpyDeviceToHost));
    return DBSN_OK;
}

int32_t dbsn_bp_steps(dbsn_mlp* m, const float* samples_dev, const int32_t* labels_dev, int64_t n, float eta,
                      float* loss_dev) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (n < 0) return fail(DBSN_E_ARG, "n is negative");
    if (n == 0) return DBSN_OK;
    if (!samples_dev || !labels_dev) return fail(DBSN_E_ARG, "samples or labels pointer is null");
    if (!aligned(samples_dev, 4) || !aligned(labels_dev, 4) || !aligned(loss_dev, 4))
        return fail(DBSN_E_SHAPE, "misaligned pointer");
    if (!std::isfinite(eta)) return fail(DBSN_E_ARG, "eta is not finite");
    if (m->mode == DBSN_MODE_PERSISTENT) return steps_persistent(m, samples_dev, labels_dev, 0, n, eta, loss_dev);
    return steps_launches(m, samples_dev, labels_dev, 0, n, eta, loss_dev);
}

int32_t dbsn_bp_step(dbsn_mlp* m, const float* sample_dev, int32_t label, float eta) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (!sample_dev) return fail(DBSN_E_ARG, "sample pointer is null");
    if (!aligned(sample_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");
    if (label < 0 || label >= m->sizes.back())
        return fail(DBSN_E_ARG, "label %d out of range 0..%d", label, m->sizes.back() - 1);
    if (!std::isfinite(eta)) return fail(DBSN_E_ARG, "eta is not finite");
    if (m->mode == DBSN_MODE_PERSISTENT) return steps_persistent(m, sample_dev, nullptr, label, 1, eta, nullptr);
    return steps_launches(m, sample_dev, nullptr, label, 1, eta, nullptr);
}

int32_t dbsn_forward(dbsn_mlp* m, const float* sample_dev, float* probs_dev) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (!sample_dev || !probs_dev) return fail(DBSN_E_ARG, "null pointer");
    if (!aligned(sample_dev, 4) || !aligned(probs_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");
    int32_t rc = forward_launches(m, sample_dev, nullptr);
    if (rc) return rc;
    HIP_TRY(hipMemcpyAsync(probs_dev, m->net.lay[m->net.L].x, sizeof(float) * m->sizes.back(),
                           hipMemcpyDeviceToDevice, m->stream));
    return DBSN_OK;
}

int32_t dbsn_classify(dbsn_mlp* m, const float* samples_dev, int64_t n, int32_t* labels_out_dev) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (n < 0) return fail(DBSN_E_ARG, "n is negative");
    if (n == 0) return DBSN_OK;
    if (!samples_dev || !labels_out_dev) return fail(DBSN_E_ARG, "null pointer");
    if (!aligned(samples_dev, 4) || !aligned(labels_out_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");
    for (int64_t s = 0; s < n; ++s) {
        int32_t rc = forward_launches(m, samples_dev + s * m->sizes[0], labels_out_dev + s);
        if (rc) return rc;
    }
    HIP_TRY(hipGetLastError());
    return DBSN_OK;
}

int32_t dbsn_deform_batch(const dbsn_deform_params* p, const uint8_t* src_dev, int64_t n, uint64_t seed,
                          uint64_t first_index, float* dst_dev, void* hip_stream) {
    if (!p) return fail(DBSN_E_ARG, "params is null");
    if (n < 0) return fail(DBSN_E_ARG, "n is negative");
    if (p->ktaps < 1 || p->ktaps > DBSN_MAX_KTAPS || (p->ktaps & 1) == 0)
        return fail(DBSN_E_ARG, "ktaps must be odd and in 1..%d", DBSN_MAX_KTAPS);
    if (!(p->sigma >= 0.0f) || !std::isfinite(p->sigma) || !std::isfinite(p->alpha) || !std::isfinite(p->beta_deg) ||
        !std::isfinite(p->gamma_pct))
        return fail(DBSN_E_ARG, "deformation parameters must be finite, sigma >= 0");
    if (n == 0) return DBSN_OK;
    if (!src_dev || !dst_dev) return fail(DBSN_E_ARG, "null pointer");
    if (!aligned(dst_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");

    DeformArgs a{};
    // 1-D Gaussian exp(-t^2 / (2 sigma^2)), t = -R..R, scaled to sum 1 (sigma 0: unit impulse)
    const int R = (p->ktaps - 1) / 2;
    double g[kMaxTaps], sum = 0.0;
    for (int t = -R; t <= R; ++t) {
        g[t + R] = (p->sigma > 0.0f) ? std::exp(-(double)(t * t) / (2.0 * (double)p->sigma * (double)p->sigma))
                                     : (t == 0 ? 1.0 : 0.0);
        sum += g[t + R];
    }
    for (int i = 0; i < p->ktaps; ++i) a.taps[i] = (float)(g[i] / sum);
    a.ktaps = p->ktaps;
    a.alpha = p->alpha;
    a.beta_deg = p->beta_deg;
    a.gamma_pct = p->gamma_pct;
    a.seed = seed;
    a.first_index = first_index;
    a.n = n;
    const int blocks = (int)(n < 65536 ? n : 65536);
    hipLaunchKernelGGL(k_deform, dim3(blocks), dim3(kDeformThreads), 0, static_cast<hipStream_t>(hip_stream), a,
                       src_dev, dst_dev);
    HIP_TRY(hipGetLastError());
    return DBSN_OK;
}

}  // extern "C"
