// libdbsn host side: the C ABI declared in include/dbsn.h.  Argument checks, arena layout,
// kernel launches.  No device memory is allocated here.
#include "dbsn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "dbsn_plan.h"
#include "dbsn_deform_kernels.h"
#include "dbsn_mlp_kernels.h"
#include "dbsn_batch_kernels.h"
#include "dbsn_persistent_kernel.h"
#include "dbsn_reduce_kernels.h"
#include "dbsn_probe_kernels.h"

using namespace dbsn;

// Staging memory of dbsn_classify_static: the two activation buffers of one batched forward pass,
// for callers that cannot allocate.  Every device the library runs on holds its own copy of the
// array until the process ends; in host code the name below is only a handle for
// hipGetSymbolAddress, the address kernels are given is the one that call returns (g_scratch_ptr).
static __device__ __align__(256) float scratch[DBSN_STATIC_SCRATCH_BYTES / sizeof(float)];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
float* g_scratch_ptr[kMaxDevices] = {};   // per device: where `scratch` lives there (null: not asked yet)

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

constexpr size_t kAlign = kArenaAlign;

// Looks up this device's copy of the static scratch array, once per device; `device` must be the
// current device.
int32_t static_scratch_setup(int device) {
    if (device < 0 || device >= kMaxDevices) return fail(DBSN_E_HIP, "device ordinal %d not supported", device);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[device]) return DBSN_OK;
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(DBSN_E_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[device] = static_cast<float*>(p);
    return DBSN_OK;
}

}  // namespace

struct dbsn_mlp {
    Net net{};
    std::vector<int32_t> sizes;
    ArenaPlan plan{};
    char* arena = nullptr;
    hipStream_t stream = nullptr;
    PNet pnet{};
    int mode = DBSN_MODE_PERSISTENT;
    int launch = DBSN_LAUNCH_COOPERATIVE;   // how the persistent kernel is launched
    uint64_t epoch = 0;        // steps run by the persistent kernel so far (its tags continue from here)
    int device = 0;
    int cus = 0;
    size_t lds_limit = 0;
    bool persistent_ready = false;   // LDS size and residency of the selected persistent kernel checked
    int layout = 0;            // register layout of the persistent kernel (0: packed at run time)
    int tiles = 0;             // which of plan.tiles the persistent kernel uses (1: the banded cut)
    bool dies_ok = false;      // the device is eight dies of 32 compute units (probed)
    unsigned die_launches = 0; // launches so far that took tickets from the per-die counters
    int* err = nullptr;
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
    const size_t lds = sizeof(float) * (size_t)phase_lds_floats(NCH);   // (registered by allow_bwd_lds at init)
    hipLaunchKernelGGL(k_bwd<NCH>, dim3(m->net.G), dim3(kThreads), lds, m->stream, m->net, l, x0, eta);
    return DBSN_OK;
}

// A backward kernel whose LDS exceeds the default limit has to be told so once.
template <int NCH>
int32_t allow_bwd_lds() {
    const size_t lds = sizeof(float) * (size_t)phase_lds_floats(NCH);
    if (lds > 64 * 1024)
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_bwd<NCH>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
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

// Two persistent kernels on the chip at once could each hold compute units the other needs for its
// last workgroups, and wait for ever (until the spin limit).  The driver keeps cooperative launches
// apart; plain ones are kept apart here, for this process: per device, the stream of the last
// persistent launch is remembered, and a launch on another stream first waits for everything that
// stream has been given so far (an event recorded on it now covers that kernel).  Same stream: in
// order anyway, nothing to do.
struct LastPersistent {
    hipStream_t stream = nullptr;
    hipEvent_t done = nullptr;
    bool any = false;
};
std::mutex g_persistent_mu;
LastPersistent g_last_persistent[kMaxDevices];

// One launch (all kPGroups workgroups resident together) runs the n steps.
int32_t steps_persistent(dbsn_mlp* m, const float* samples, const int* labels, int label_val, int64_t n, float eta,
                         float* loss) {
    const size_t lds = sizeof(float) * (size_t)(PLds::total + kProfLdsFloats);
    const void* fn = !m->pnet.stationary ? reinterpret_cast<const void*>(&k_bp_dataflow<false, 0>)
                     : m->layout == 1    ? reinterpret_cast<const void*>(&k_bp_dataflow<true, 1>)
                     : m->layout == 2    ? reinterpret_cast<const void*>(&k_bp_dataflow<true, 2>)
                     : m->layout == 3    ? reinterpret_cast<const void*>(&k_bp_dataflow<true, 3>)
                                         : reinterpret_cast<const void*>(&k_bp_dataflow<true, 0>);
    if (!m->persistent_ready) {
        if (lds > m->lds_limit) return fail(DBSN_E_SHAPE, "persistent kernel needs %zu B of LDS", lds);
        HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        int per_cu = 0;
        HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kThreads, lds));
        if (per_cu * m->cus < kPGroups)
            return fail(DBSN_E_SHAPE, "device cannot hold %d resident workgroups", kPGroups);
        m->persistent_ready = true;
    }
    PNet net = m->pnet;
    long long nn = n;
    unsigned base = (unsigned)m->epoch;
    unsigned seq = m->die_launches;   // launches that took tickets so far: this one's tickets start at 32 * seq per die
    void* args[] = {&net, &samples, &labels, &label_val, &nn, &eta, &loss, &base, &seq};
    {
        std::lock_guard<std::mutex> lock(g_persistent_mu);
        LastPersistent& last = g_last_persistent[m->device];
        if (last.any && last.stream != m->stream) {
            if (!last.done) HIP_TRY(hipEventCreateWithFlags(&last.done, hipEventDisableTiming));
            if (hipEventRecord(last.done, last.stream) == hipSuccess) {
                HIP_TRY(hipStreamWaitEvent(m->stream, last.done, 0));
            } else {   // (that stream is gone: wait for the device instead)
                (void)hipGetLastError();
                HIP_TRY(hipDeviceSynchronize());
            }
        }
        if (m->launch == DBSN_LAUNCH_PLAIN)
            HIP_TRY(hipLaunchKernel(fn, dim3(kPGroups), dim3(kThreads), args, (unsigned)lds, m->stream));
        else
            HIP_TRY(hipLaunchCooperativeKernel(fn, dim3(kPGroups), dim3(kThreads), args, (unsigned)lds, m->stream));
        last.any = true;
        last.stream = m->stream;
    }
    if (net.any_local) ++m->die_launches;
    m->epoch += (uint64_t)n;
    return DBSN_OK;
}

// Fills the persistent kernel's view of the network for the chosen variant: weights stationary in
// registers or streamed per phase; row slots in a compile-time layout or packed at run time; tiles
// in the banded cut (hand-overs inside a die where the layers pair up) or the plain one.
void configure_persistent(dbsn_mlp* m, bool stationary, bool fixed_layout, bool banded) {
    const ArenaPlan& plan = m->plan;
    const Net& net = m->net;
    PNet& pn = m->pnet;
    m->tiles = (banded && plan.banded && m->dies_ok) ? 1 : 0;
    const TilePlan& tp = plan.tiles[m->tiles];
    pn.stationary = (stationary && tp.stationary) ? 1 : 0;
    m->layout = (pn.stationary && fixed_layout) ? choose_layout(tp, net.L) : 0;
    pn.any_local = 0;
    for (int l = 1; l <= net.L; ++l) {
        PLayer& P = pn.lay[l];
        const Layer& Ly = net.lay[l];
        P = PLayer{};
        P.W = Ly.W; P.b = Ly.b; P.x = Ly.x; P.d = Ly.d;
        P.n_in = Ly.n_in; P.n_out = Ly.n_out; P.ld = Ly.ld;
        if (l < net.L && tp.ok) {
            P.shape = tp.shape[l];
            P.s0 = m->layout ? kLayoutS0[m->layout][l - 1] : (pn.stationary ? tp.s0[l] : 0);
            P.ns = tp.ns[l];
            P.fwd_local = tp.fwd_local[l] ? 1 : 0;
            P.bwd_local = tp.bwd_local[l] ? 1 : 0;
            pn.any_local |= P.fwd_local | P.bwd_local;
            P.yp = reinterpret_cast<u64*>(m->arena + plan.yp[l]);
            if (l <= net.L - 2) {
                P.gp = reinterpret_cast<u64*>(m->arena + plan.gp[l]);
                P.gP = tp.gP[l];
            }
        }
    }
    m->persistent_ready = false;
}

// Is the device eight dies that take 32 workgroups of the training kernel each?  Asked once per
// device: a small kernel of the same launch shape notes the die every workgroup finds itself on
// (in the static scratch array).
std::mutex g_dies_mu;
int g_dies_state[kMaxDevices] = {};   // 0: not probed, 1: yes, 2: no
bool device_has_eight_dies(int device, hipStream_t stream) {
    std::lock_guard<std::mutex> lock(g_dies_mu);
    if (device < 0 || device >= kMaxDevices) return false;
    if (g_dies_state[device] == 0) {
        g_dies_state[device] = 2;
        int* ids = nullptr;
        {
            std::lock_guard<std::mutex> lk(g_scratch_mu);
            ids = reinterpret_cast<int*>(g_scratch_ptr[device]);
        }
        int host[kPGroups];
        if (ids) {
            const size_t lds = sizeof(float) * (size_t)(PLds::total + kProfLdsFloats);   // the training kernel's footprint: one workgroup per CU
            const void* fn = reinterpret_cast<const void*>(&k_die_probe);
            void* args[] = {&ids};
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
                hipLaunchCooperativeKernel(fn, dim3(kPGroups), dim3(kThreads), args, (unsigned)lds, stream) == hipSuccess &&
                hipStreamSynchronize(stream) == hipSuccess &&
                hipMemcpy(host, ids, sizeof host, hipMemcpyDeviceToHost) == hipSuccess) {
                int per_die[kXcds] = {};
                bool ok = true;
                for (int g = 0; g < kPGroups; ++g) {
                    ok = ok && host[g] >= 0 && host[g] < kXcds;
                    if (ok) ++per_die[host[g]];
                }
                for (int k = 0; k < kXcds; ++k) ok = ok && per_die[k] == kPGroups / kXcds;
                if (ok) g_dies_state[device] = 1;
            }
            (void)hipGetLastError();
        }
    }
    return g_dies_state[device] == 1;
}

// (the persistent kernel needs all its workgroups resident at once, one per compute unit)
bool use_persistent(const dbsn_mlp* m) {
    return m->mode == DBSN_MODE_PERSISTENT && m->plan.persistent_ok && m->cus >= kPGroups;
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
    if (int32_t rc = static_scratch_setup(m->device)) {
        delete m;
        return rc;
    }
    m->lds_limit = prop.sharedMemPerBlock;
    m->cus = prop.multiProcessorCount;
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
    }
    net.gpart[0] = reinterpret_cast<float*>(m->arena + plan.gpart[0]);
    net.gpart[1] = reinterpret_cast<float*>(m->arena + plan.gpart[1]);
    m->err = reinterpret_cast<int*>(m->arena + plan.flags);

    PNet& pn = m->pnet;
    pn.L = net.L;
    pn.err = m->err;
    pn.spin_limit = 1u << 22;
    // pauses before the first look at the partial sums of a phase, in units of 64 clocks: forward
    // consumers arrive about half a microsecond before the other tiles' words are visible, backward
    // ones late enough by themselves (dbsn_mlp_autotune / dbsn_mlp_set_pauses refine them)
    for (int l = 0; l <= kMaxLayers; ++l) {
        pn.pace[0][l] = 17;
        pn.pace[1][l] = 0;
    }
    m->dies_ok = plan.banded && prop.multiProcessorCount == kPGroups && device_has_eight_dies(m->device, m->stream);
    configure_persistent(m, true, true, true);
    // (a hand-over inside a die is there sooner: the layers that read one look earlier)
    for (int l = 2; l < net.L; ++l)
        if (pn.lay[l].bwd_local) pn.pace[0][l] = 2;
    // kernels that need more LDS than the default limit say so once, here
    {
        int32_t rc = DBSN_OK;
        for (int l = 1; l < net.L && !rc; ++l) {
            rc = DBSN_E_SHAPE;
            DBSN_NCH_SWITCH(16, net.lay[l].nch, rc = allow_bwd_lds<N>());
        }
        if (!rc && hipFuncSetAttribute(reinterpret_cast<const void*>(&k_layer_batch_dma<true, 128>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)dma_lds_bytes(128)) != hipSuccess)
            rc = fail(DBSN_E_HIP, "hipFuncSetAttribute(k_layer_batch_dma<128>)");
        if (!rc && hipFuncSetAttribute(reinterpret_cast<const void*>(&k_layer_batch_dma<true, 64>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)dma_lds_bytes(64)) != hipSuccess)
            rc = fail(DBSN_E_HIP, "hipFuncSetAttribute(k_layer_batch_dma<64>)");
        if (rc) {
            delete m;
            return rc == DBSN_E_SHAPE ? fail(rc, "unsupported layer width") : rc;
        }
    }

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
    {   // (nothing of this stream is running any more: no later launch needs to wait for it)
        std::lock_guard<std::mutex> lock(g_persistent_mu);
        LastPersistent& last = g_last_persistent[m->device];
        if (last.any && last.stream == m->stream) last.any = false;
    }
    delete m;
    return DBSN_OK;
}

int32_t dbsn_mlp_set_mode(dbsn_mlp* m, int32_t mode) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (mode != DBSN_MODE_LAUNCHES && mode != DBSN_MODE_PERSISTENT) return fail(DBSN_E_ARG, "unknown mode %d", mode);
    m->mode = mode;
    return DBSN_OK;
}

int32_t dbsn_mlp_set_launch(dbsn_mlp* m, int32_t kind) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (kind != DBSN_LAUNCH_COOPERATIVE && kind != DBSN_LAUNCH_PLAIN) return fail(DBSN_E_ARG, "unknown launch kind %d", kind);
    m->launch = kind;
    return DBSN_OK;
}

int32_t dbsn_mlp_set_spin_limit(dbsn_mlp* m, uint32_t polls) {
    if (check_mlp(m)) return DBSN_E_ARG;
    m->pnet.spin_limit = polls;
    return DBSN_OK;
}

int32_t dbsn_mlp_set_pauses(dbsn_mlp* m, const int32_t* fwd_host, const int32_t* bwd_host) {
    if (check_mlp(m)) return DBSN_E_ARG;
    const int L = m->net.L;
    for (int dir = 0; dir < 2; ++dir) {
        const int32_t* src = dir == 0 ? fwd_host : bwd_host;
        if (!src) continue;
        for (int l = 1; l <= L; ++l)
            if (src[l - 1] < 0 || src[l - 1] > kPaceMax)
                return fail(DBSN_E_ARG, "pause %d of layer %d outside 0..%d", src[l - 1], l, kPaceMax);
    }
    for (int dir = 0; dir < 2; ++dir) {
        const int32_t* src = dir == 0 ? fwd_host : bwd_host;
        if (!src) continue;
        for (int l = 1; l <= L; ++l) m->pnet.pace[dir][l] = (unsigned char)src[l - 1];
    }
    return DBSN_OK;
}

int32_t dbsn_mlp_get_pauses(dbsn_mlp* m, int32_t* fwd_host, int32_t* bwd_host) {
    if (check_mlp(m)) return DBSN_E_ARG;
    for (int l = 1; l <= m->net.L; ++l) {
        if (fwd_host) fwd_host[l - 1] = m->pnet.pace[0][l];
        if (bwd_host) bwd_host[l - 1] = m->pnet.pace[1][l];
    }
    return DBSN_OK;
}

int32_t dbsn_mlp_set_variant(dbsn_mlp* m, int32_t stationary, int32_t fixed_layout, int32_t banded) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if ((stationary != 0 && stationary != 1) || (fixed_layout != 0 && fixed_layout != 1) || (banded != 0 && banded != 1))
        return fail(DBSN_E_ARG, "stationary, fixed_layout and banded must be 0 or 1");
    HIP_TRY(hipStreamSynchronize(m->stream));
    configure_persistent(m, stationary != 0, fixed_layout != 0, banded != 0);
    return DBSN_OK;
}

int32_t dbsn_mlp_get_variant(dbsn_mlp* m, int32_t* stationary, int32_t* layout, int32_t* banded_pairs) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (stationary) *stationary = m->pnet.stationary;
    if (layout) *layout = m->layout;
    if (banded_pairs) *banded_pairs = m->tiles ? m->plan.tiles[1].pairs : 0;
    return DBSN_OK;
}

int32_t dbsn_mlp_status(dbsn_mlp* m) {
    if (check_mlp(m)) return DBSN_E_ARG;
    HIP_TRY(hipStreamSynchronize(m->stream));
    int err = 0;
    HIP_TRY(hipMemcpy(&err, m->err, sizeof err, hipMemcpyDeviceToHost));
    if (err == 2) {
        HIP_TRY(hipMemset(m->err, 0, sizeof(int)));
        m->epoch += (uint64_t)1 << 20;
        m->dies_ok = false;   // fall back to the plain cut from here on
        configure_persistent(m, m->pnet.stationary != 0, m->layout != 0, false);
        return fail(DBSN_E_HIP, "the workgroups of a launch did not come 32 to a die; the banded tiles are switched off, "
                                "the weights are undefined");
    }
    if (err) {
        HIP_TRY(hipMemset(m->err, 0, sizeof(int)));
        // stale partial sums of the abandoned steps must never match a later step's tag
        m->epoch += (uint64_t)1 << 20;
        return fail(DBSN_E_TIMEOUT, "a wait inside the persistent kernel gave up; weights are undefined");
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
    if (use_persistent(m)) return steps_persistent(m, samples_dev, labels_dev, 0, n, eta, loss_dev);
    return steps_launches(m, samples_dev, labels_dev, 0, n, eta, loss_dev);
}

int32_t dbsn_mlp_autotune(dbsn_mlp* m, const float* samples_dev, const int32_t* labels_dev, int64_t n) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (n < 64) return fail(DBSN_E_ARG, "autotune needs at least 64 samples");
    if (!samples_dev || !labels_dev) return fail(DBSN_E_ARG, "samples or labels pointer is null");
    if (!aligned(samples_dev, 4) || !aligned(labels_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");
    if (!use_persistent(m)) return DBSN_OK;   // the launch-per-phase mode has nothing to tune
    // Coordinate descent over the pauses of the persistent kernel, timing launches of steps with
    // eta = 0: w - 0 * delta * x is w, bit for bit, so the weights come out as they went in.
    const int64_t steps = std::min<int64_t>(n, 512);
    const int L = m->net.L;
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail(DBSN_E_HIP, "hipEventCreate");
    }
    int32_t rc = DBSN_OK;
    auto measure = [&](float& best_ms) -> int32_t {
        best_ms = 1e30f;
        for (int rep = 0; rep < 3; ++rep) {
            if (hipEventRecord(e0, m->stream) != hipSuccess) return fail(DBSN_E_HIP, "hipEventRecord");
            const int32_t r = steps_persistent(m, samples_dev, labels_dev, 0, steps, 0.0f, nullptr);
            if (r) return r;
            if (hipEventRecord(e1, m->stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess)
                return fail(DBSN_E_HIP, "hipEventSynchronize");
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return fail(DBSN_E_HIP, "hipEventElapsedTime");
            best_ms = std::min(best_ms, ms);
        }
        return DBSN_OK;
    };
    float best = 0.0f;
    rc = measure(best);   // (also warms the launch up)
    if (!rc) rc = measure(best);
    const int coarse[] = {-4, -2, 2, 4, 8}, fine[] = {-1, 1};
    for (int sweep = 0; sweep < 2 && !rc; ++sweep) {
        const int* deltas = sweep == 0 ? coarse : fine;
        const int nd = sweep == 0 ? 5 : 2;
        for (int dir = 0; dir < 2 && !rc; ++dir)
            for (int l = 1; l <= L && !rc; ++l) {
                unsigned char& cell = m->pnet.pace[dir][l];
                int base = cell;
                for (int k = 0; k < nd && !rc; ++k) {
                    const int v = base + deltas[k];
                    if (v < 0 || v > 48) continue;
                    cell = (unsigned char)v;
                    float ms = 0.0f;
                    rc = measure(ms);
                    if (!rc && ms < best * 0.9985f) {   // keep what is better by more than the noise
                        best = ms;
                        base = v;
                    }
                    cell = (unsigned char)base;
                }
            }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    return dbsn_mlp_status(m);
}

int32_t dbsn_bp_step(dbsn_mlp* m, const float* sample_dev, int32_t label, float eta) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (!sample_dev) return fail(DBSN_E_ARG, "sample pointer is null");
    if (!aligned(sample_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");
    if (label < 0 || label >= m->sizes.back())
        return fail(DBSN_E_ARG, "label %d out of range 0..%d", label, m->sizes.back() - 1);
    if (!std::isfinite(eta)) return fail(DBSN_E_ARG, "eta is not finite");
    if (use_persistent(m)) return steps_persistent(m, sample_dev, nullptr, label, 1, eta, nullptr);
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

}  // extern "C"

namespace {

// The batched forward pass over n samples, `per` at a time: one launch per layer, the activations
// of a pass alternating between the two buffers act[0] and act[1] ([per][ldact] floats each).
int32_t classify_passes(dbsn_mlp* m, const float* samples_dev, int64_t n, int32_t* labels_out_dev, float* const act[2],
                        int64_t per) {
    const int L = m->net.L, n0 = m->sizes[0], ldact = m->plan.ldact;
    for (int64_t at = 0; at < n; at += per) {
        const int S = (int)std::min<int64_t>(per, n - at);
        const float* X = samples_dev + at * n0;
        int ldx = n0;
        for (int l = 1; l < L; ++l) {
            const Layer& Ly = m->net.lay[l];
            float* Y = act[l & 1];
            const dim3 grid((Ly.n_out + kBatchTile - 1) / kBatchTile, (S + kBatchTile - 1) / kBatchTile);
            // the fast kernel when every operand row starts on a 16-byte boundary and holds a whole
            // number of float4 (always true of the activation buffers; of the caller's samples and
            // the first layer when sizes[0] % 4 == 0), else the kernel that stages by element
            // (and when its 32-bit byte offsets reach every element)
            const bool fits = (uint64_t)Ly.n_out * Ly.ld * sizeof(float) < (1ull << 32) &&
                              (uint64_t)S * std::max(ldx, ldact) * sizeof(float) < (1ull << 32);
            if (fits && ldx % 4 == 0 && Ly.ld % 4 == 0 && Ly.n_in % 4 == 0 && aligned(X, 16) && aligned(Ly.W, 16)) {
                // tiles of 128 samples, or of 64 where that fills the rounds of the persistent
                // workgroups better: a 64-sample tile costs a little more than half a 128-sample one
                const int nx = (int)grid.x, G = m->cus;
                const int nt128 = nx * ((S + 127) / 128), nt64 = nx * ((S + 63) / 64);
                const double cost128 = (double)((nt128 + G - 1) / G), cost64 = 0.54 * (double)((nt64 + G - 1) / G);
                const float* zeros = reinterpret_cast<const float*>(m->err + kZerosAt);
                if (cost64 < cost128)
                    hipLaunchKernelGGL((k_layer_batch_dma<true, 64>), dim3(std::min(nt64, G)), dim3(kDmaThreads),
                                       dma_lds_bytes(64), m->stream, X, ldx, S, Ly.W, Ly.ld, Ly.b, Ly.n_in, Ly.n_out, Y,
                                       ldact, nx, nt64, zeros);
                else
                    hipLaunchKernelGGL((k_layer_batch_dma<true, 128>), dim3(std::min(nt128, G)), dim3(kDmaThreads),
                                       dma_lds_bytes(128), m->stream, X, ldx, S, Ly.W, Ly.ld, Ly.b, Ly.n_in, Ly.n_out, Y,
                                       ldact, nx, nt128, zeros);
            } else {
                hipLaunchKernelGGL(k_layer_batch<true>, grid, dim3(kBatchThreads), 0, m->stream, X, ldx, S, Ly.W,
                                   Ly.ld, Ly.b, Ly.n_in, Ly.n_out, Y, ldact);
            }
            X = Y;
            ldx = ldact;
        }
        const Layer& Lt = m->net.lay[L];
        if (ldx % 4 == 0 && Lt.ld % 4 == 0 && aligned(X, 16) && aligned(Lt.W, 16)) {
            const int per_block = (kBatchThreads / 64) * kTopPerWave;
            hipLaunchKernelGGL(k_top_batch, dim3((S + per_block - 1) / per_block), dim3(kBatchThreads), 0, m->stream, X,
                               ldx, S, Lt.W, Lt.ld, Lt.b, Lt.n_in, Lt.n_out, labels_out_dev + at);
        } else {
            const int per_block = kBatchThreads / 64;
            hipLaunchKernelGGL(k_top_batch_any, dim3((S + per_block - 1) / per_block), dim3(kBatchThreads), 0, m->stream,
                               X, ldx, S, Lt.W, Lt.ld, Lt.b, Lt.n_in, Lt.n_out, labels_out_dev + at);
        }
    }
    HIP_TRY(hipGetLastError());
    return DBSN_OK;
}

int32_t check_classify_args(dbsn_mlp* m, const float* samples_dev, int64_t n, const int32_t* labels_out_dev) {
    if (check_mlp(m)) return DBSN_E_ARG;
    if (n < 0) return fail(DBSN_E_ARG, "n is negative");
    if (n > 0 && (!samples_dev || !labels_out_dev)) return fail(DBSN_E_ARG, "null pointer");
    if (!aligned(samples_dev, 4) || !aligned(labels_out_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");
    return DBSN_OK;
}

}  // namespace

extern "C" {

int32_t dbsn_classify(dbsn_mlp* m, const float* samples_dev, int64_t n, int32_t* labels_out_dev) {
    if (int32_t rc = check_classify_args(m, samples_dev, n, labels_out_dev)) return rc;
    if (n == 0) return DBSN_OK;
    // the samples go through the layers in passes of kBatchSamples (what the arena's buffers hold)
    float* const act[2] = {reinterpret_cast<float*>(m->arena + m->plan.act[0]),
                           reinterpret_cast<float*>(m->arena + m->plan.act[1])};
    return classify_passes(m, samples_dev, n, labels_out_dev, act, kBatchSamples);
}

int32_t dbsn_classify_static(dbsn_mlp* m, const float* samples_dev, int64_t n, int32_t* labels_out_dev) {
    if (int32_t rc = check_classify_args(m, samples_dev, n, labels_out_dev)) return rc;
    if (n == 0) return DBSN_OK;
    // one pass: both activation buffers of all n samples must fit the static array
    const size_t row = sizeof(float) * (size_t)m->plan.ldact;
    const size_t half = DBSN_STATIC_SCRATCH_BYTES / 2;
    if ((uint64_t)n > half / row)
        return fail(DBSN_E_SHAPE, "n = %lld is beyond the static scratch: at most %zu samples per call for a widest "
                                  "layer of %d neurons (2 x n x %zu bytes <= %zu)",
                    (long long)n, half / row, m->plan.ldact, row, (size_t)DBSN_STATIC_SCRATCH_BYTES);
    float* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        base = g_scratch_ptr[m->device];
    }
    if (!base) return fail(DBSN_E_HIP, "static scratch of device %d was not set up", m->device);
    float* const act[2] = {base, base + half / sizeof(float)};
    // The array keeps what the last call left (possibly of another network).  The kernels read a few
    // columns past a layer's outputs against zero weights, so what they find there must be finite:
    // both regions start at zero, by a kernel (no memset, which callers recording a graph avoid).
    const long long n4 = (long long)((size_t)n * row / sizeof(float4));
    const int blocks = (int)std::min<long long>((n4 + 255) / 256, 2048);
    hipLaunchKernelGGL(k_zero, dim3(blocks), dim3(256), 0, m->stream, reinterpret_cast<float4*>(act[0]), n4);
    hipLaunchKernelGGL(k_zero, dim3(blocks), dim3(256), 0, m->stream, reinterpret_cast<float4*>(act[1]), n4);
    return classify_passes(m, samples_dev, n, labels_out_dev, act, n);
}

}  // extern "C"

namespace {

// Checks and launch shared by the three deformation calls: at most one of beta_each / labels is set.
int32_t deform_launch(const dbsn_deform_params* p, const uint8_t* src_dev, const float* beta_deg_dev,
                      const int32_t* labels_dev, uint64_t similar_mask, float beta_similar_deg, int64_t n,
                      uint64_t seed, uint64_t first_index, float* dst_dev, void* hip_stream) {
    if (!p) return fail(DBSN_E_ARG, "params is null");
    if (n < 0) return fail(DBSN_E_ARG, "n is negative");
    if (p->ktaps < 1 || p->ktaps > DBSN_MAX_KTAPS || (p->ktaps & 1) == 0)
        return fail(DBSN_E_ARG, "ktaps must be odd and in 1..%d", DBSN_MAX_KTAPS);
    if (!(p->sigma >= 0.0f) || !std::isfinite(p->sigma) || !std::isfinite(p->alpha) || !std::isfinite(p->beta_deg) ||
        !std::isfinite(p->gamma_pct) || !std::isfinite(beta_similar_deg))
        return fail(DBSN_E_ARG, "deformation parameters must be finite, sigma >= 0");
    if (p->shear != 0 && p->shear != 1) return fail(DBSN_E_ARG, "shear must be 0 or 1");
    if (p->kernel != DBSN_DEFORM_KERNEL_AUTO && p->kernel != DBSN_DEFORM_KERNEL_GENERAL)
        return fail(DBSN_E_ARG, "kernel must be DBSN_DEFORM_KERNEL_AUTO or DBSN_DEFORM_KERNEL_GENERAL");
    if (n == 0) return DBSN_OK;
    if (!src_dev || !dst_dev) return fail(DBSN_E_ARG, "null pointer");
    if (!aligned(dst_dev, 4) || !aligned(beta_deg_dev, 4) || !aligned(labels_dev, 4))
        return fail(DBSN_E_SHAPE, "misaligned pointer");

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
    a.shear = p->shear;
    a.beta_each = beta_deg_dev;
    a.labels = labels_dev;
    a.similar_mask = similar_mask;
    a.beta_similar = beta_similar_deg;
    a.seed = seed;
    a.first_index = first_index;
    a.n = n;
    const int blocks = (int)(n < 65536 ? n : 65536);
    // the paper's 21 taps have a kernel of their own, same results bit for bit
    if (p->ktaps == 21 && p->kernel == DBSN_DEFORM_KERNEL_AUTO)
        hipLaunchKernelGGL(k_deform_taps<21>, dim3(blocks), dim3(kDeformThreads), 0, static_cast<hipStream_t>(hip_stream),
                           a, src_dev, dst_dev);
    else
        hipLaunchKernelGGL(k_deform, dim3(blocks), dim3(kDeformThreads), 0, static_cast<hipStream_t>(hip_stream), a,
                           src_dev, dst_dev);
    HIP_TRY(hipGetLastError());
    return DBSN_OK;
}

}  // namespace

extern "C" {

int32_t dbsn_deform_batch(const dbsn_deform_params* p, const uint8_t* src_dev, int64_t n, uint64_t seed,
                          uint64_t first_index, float* dst_dev, void* hip_stream) {
    return deform_launch(p, src_dev, nullptr, nullptr, 0, 0.0f, n, seed, first_index, dst_dev, hip_stream);
}

int32_t dbsn_deform_batch_beta(const dbsn_deform_params* p, const uint8_t* src_dev, const float* beta_deg_dev,
                               int64_t n, uint64_t seed, uint64_t first_index, float* dst_dev, void* hip_stream) {
    if (n > 0 && !beta_deg_dev) return fail(DBSN_E_ARG, "beta_deg_dev is null");
    return deform_launch(p, src_dev, beta_deg_dev, nullptr, 0, 0.0f, n, seed, first_index, dst_dev, hip_stream);
}

int32_t dbsn_deform_batch_labels(const dbsn_deform_params* p, const uint8_t* src_dev, const int32_t* labels_dev,
                                 uint64_t similar_mask, float beta_similar_deg, int64_t n, uint64_t seed,
                                 uint64_t first_index, float* dst_dev, void* hip_stream) {
    if (n > 0 && !labels_dev) return fail(DBSN_E_ARG, "labels_dev is null");
    return deform_launch(p, src_dev, nullptr, labels_dev, similar_mask, beta_similar_deg, n, seed, first_index, dst_dev,
                         hip_stream);
}

int32_t dbsn_count_errors(const int32_t* predicted_dev, const int32_t* labels_dev, int64_t n, int64_t* count_dev,
                          void* hip_stream) {
    if (n < 0) return fail(DBSN_E_ARG, "n is negative");
    if (!count_dev) return fail(DBSN_E_ARG, "count_dev is null");
    if (n > 0 && (!predicted_dev || !labels_dev)) return fail(DBSN_E_ARG, "null pointer");
    if (!aligned(predicted_dev, 4) || !aligned(labels_dev, 4) || !aligned(count_dev, 8))
        return fail(DBSN_E_SHAPE, "misaligned pointer");
    hipLaunchKernelGGL(k_count_errors, dim3(1), dim3(kReduceThreads), 0, static_cast<hipStream_t>(hip_stream),
                       predicted_dev, labels_dev, (long long)n, reinterpret_cast<long long*>(count_dev));
    HIP_TRY(hipGetLastError());
    return DBSN_OK;
}

int32_t dbsn_probe_stream(float* buf_dev, int64_t n_floats, int32_t workgroups, int32_t sweeps, float* sink_dev,
                          void* hip_stream) {
    if (!buf_dev || !sink_dev) return fail(DBSN_E_ARG, "null pointer");
    if (n_floats < 4 || n_floats % 4 != 0) return fail(DBSN_E_ARG, "n_floats must be a positive multiple of 4");
    if (workgroups < 1 || workgroups > 65536) return fail(DBSN_E_ARG, "workgroups must be in 1..65536");
    if (sweeps < 0) return fail(DBSN_E_ARG, "sweeps is negative");
    if (!aligned(buf_dev, 16) || !aligned(sink_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    for (int r = 0; r < sweeps; ++r) {
        hipLaunchKernelGGL(k_probe_read, dim3(workgroups), dim3(kProbeThreads), 0, st,
                           reinterpret_cast<const float4*>(buf_dev), (long long)(n_floats / 4), sink_dev);
        hipLaunchKernelGGL(k_probe_update, dim3(workgroups), dim3(kProbeThreads), 0, st,
                           reinterpret_cast<float4*>(buf_dev), (long long)(n_floats / 4), 0.0f);
    }
    HIP_TRY(hipGetLastError());
    return DBSN_OK;
}

int32_t dbsn_probe_handover(int32_t within_die, int32_t rounds, uint64_t* buf_dev, int32_t* gave_up_dev, void* hip_stream) {
    if (!buf_dev || !gave_up_dev) return fail(DBSN_E_ARG, "null pointer");
    if (within_die != 0 && within_die != 1) return fail(DBSN_E_ARG, "within_die must be 0 or 1");
    if (rounds < 0 || rounds > (1 << 24)) return fail(DBSN_E_ARG, "rounds must be in 0..2^24");
    if (!aligned(buf_dev, 8) || !aligned(gave_up_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    unsigned long long* buf = reinterpret_cast<unsigned long long*>(buf_dev);
    unsigned limit = 1u << 16;
    // the buffer and the counter start at zero (by a kernel: callers may be recording a graph)
    const long long n4 = (long long)(2 * kHandoverGroups * kHandoverWords * sizeof(uint64_t) / sizeof(float4));
    hipLaunchKernelGGL(k_zero, dim3(64), dim3(256), 0, st, reinterpret_cast<float4*>(buf_dev), n4);
    hipLaunchKernelGGL(k_zero_int, dim3(1), dim3(64), 0, st, gave_up_dev, 1);
    const void* fn = within_die ? reinterpret_cast<const void*>(&k_probe_handover<true>)
                                : reinterpret_cast<const void*>(&k_probe_handover<false>);
    void* args[] = {&buf, &rounds, &limit, &gave_up_dev};
    HIP_TRY(hipLaunchCooperativeKernel(fn, dim3(kHandoverGroups), dim3(64), args, 0, st));
    return DBSN_OK;
}

int32_t dbsn_mean_loss(const float* loss_dev, int64_t n, float* mean_dev, void* hip_stream) {
    if (n < 1) return fail(DBSN_E_ARG, "n must be at least 1");
    if (!loss_dev || !mean_dev) return fail(DBSN_E_ARG, "null pointer");
    if (!aligned(loss_dev, 4) || !aligned(mean_dev, 4)) return fail(DBSN_E_SHAPE, "misaligned pointer");
    hipLaunchKernelGGL(k_mean, dim3(1), dim3(kReduceThreads), 0, static_cast<hipStream_t>(hip_stream), loss_dev,
                       (long long)n, mean_dev);
    HIP_TRY(hipGetLastError());
    return DBSN_OK;
}

}  // extern "C"
