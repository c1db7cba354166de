/*
 * dbsn_oracle — plain, slow, obviously-correct CPU reference for on-line
 * back-propagation through plain MLPs and for elastic + affine image
 * deformation, after Ciresan, Meier, Gambardella, Schmidhuber, "Deep Big
 * Simple Neural Nets Excel on Handwritten Digit Recognition".
 *
 * THIS IS TEST INFRASTRUCTURE. Only the test-suite, the smoke check and the
 * CPU-baseline leg of the benchmark may call it.  It shares no code, header,
 * table or constant generator with the GPU library; the GPU library never
 * links or loads it.
 *
 * Everything is written as the definition reads: scalar loops, sums taken
 * left to right, no blocking, no fusion.  Every routine exists twice, once
 * with every variable `float` (suffix _f32, libm float routines) and once
 * with every variable `double` (suffix _f64).
 *
 * Parameter packing used by every MLP routine here: for layer l = 1..L
 * (L = n_sizes-1) the dense row-major matrix W_l[n_l][n_{l-1}] followed by
 * the bias vector b_l[n_l]; layers are concatenated in order.
 *
 * Optional OpenMP: only loops whose iterations are independent (one output
 * neuron / one input column / one image per iteration) are split; the order
 * of every floating-point sum is the same for any thread count.
 */
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

int g_threads = 1;

/* ------------------------------------------------------------------------
 * Counter-based random numbers (the paper names no generator; this one is
 * this project's own definition).
 *   mix(z)      : the SplitMix64 output function (Steele, Lea, Flood 2014)
 *   key(seed,s) : mix(seed + (s+1)*GOLD)       -- s-th SplitMix64 output
 *   draw(c)     : mix(key + (c+1)*GOLD)        -- c-th output from state key
 *   sym(r)      : ((r >> 40) - 2^23) * 2^-23   in [-1, 1), exact in float
 * ---------------------------------------------------------------------- */
const uint64_t GOLD = 0x9E3779B97F4A7C15ull;

uint64_t mix(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}
uint64_t stream_key(uint64_t seed, uint64_t stream) { return mix(seed + (stream + 1) * GOLD); }
uint64_t draw(uint64_t key, uint64_t counter) { return mix(key + (counter + 1) * GOLD); }
float sym_unit(uint64_t r) {
    int32_t k = (int32_t)(r >> 40) - (1 << 23);          /* -2^23 .. 2^23-1 */
    return (float)k * (1.0f / 8388608.0f);               /* exact: one power-of-two scale */
}

/* ------------------------------------------------------------------------
 * Activation (section "Architectures"): y(a) = A tanh(B a), A = 1.7159,
 * B = 0.6666 as printed.  The derivative is taken from the stored output y,
 * as the delta back-propagation of the appendix does:
 *   dy/da = A B (1 - tanh^2(B a)) = (B/A) (A^2 - y^2).
 * ---------------------------------------------------------------------- */
template <class T> struct K;
template <> struct K<float>  { static float  A() { return 1.7159f; } static float  B() { return 0.6666f; } };
template <> struct K<double> { static double A() { return 1.7159;  } static double B() { return 0.6666;  } };

template <class T> T act(T a) { return K<T>::A() * std::tanh(K<T>::B() * a); }
template <class T> T dact_from_y(T y) { return (K<T>::B() / K<T>::A()) * (K<T>::A() * K<T>::A() - y * y); }

int64_t param_count(const int32_t* sizes, int32_t n_sizes) {
    int64_t n = 0;
    for (int l = 1; l < n_sizes; ++l) n += (int64_t)(sizes[l - 1] + 1) * sizes[l];
    return n;
}

/* Forward propagation (appendix "Forward propagation" for the hidden layers;
 * the 10-way softmax output is the reading fixed for this project, the paper
 * does not name its output non-linearity).
 * acts: x_1 .. x_{L-1} concatenated, then the L-th layer's pre-activations
 * (logits); probs: softmax of the logits. */
template <class T>
void forward(const int32_t* sizes, int32_t n_sizes, const T* params, const T* x0, T* acts, T* probs) {
    const int L = n_sizes - 1;
    const T* xin = x0;
    const T* p = params;
    T* out = acts;
    for (int l = 1; l <= L; ++l) {
        const int nin = sizes[l - 1], nout = sizes[l];
        const T* W = p;
        const T* b = p + (int64_t)nin * nout;
#pragma omp parallel for num_threads(g_threads) if (g_threads > 1)
        for (int j = 0; j < nout; ++j) {
            T a = b[j];
            for (int i = 0; i < nin; ++i) a += W[(int64_t)j * nin + i] * xin[i];
            out[j] = (l < L) ? act<T>(a) : a;
        }
        p += (int64_t)(nin + 1) * nout;
        xin = out;
        out += nout;
    }
    /* softmax with the usual max shift */
    const int nc = sizes[L];
    const T* a = xin;
    T m = a[0];
    for (int k = 1; k < nc; ++k) if (a[k] > m) m = a[k];
    T s = 0;
    for (int k = 0; k < nc; ++k) { probs[k] = std::exp(a[k] - m); s += probs[k]; }
    for (int k = 0; k < nc; ++k) probs[k] = probs[k] / s;
}

/* One on-line back-propagation step on one sample (sections "Architectures"
 * and "Training algorithm", appendix "Backward propagation" and "Weight
 * updating"): all deltas are obtained from the weights as they were before
 * the step; only then is a weight changed: w_ji -= eta * delta_j * x_i, the
 * bias being the weight of a constant-1 input.  No momentum, batch size 1.
 * deltas_out (nullable): delta_1 .. delta_L concatenated. */
template <class T>
T bp_step(const int32_t* sizes, int32_t n_sizes, T* params, const T* x0, int32_t label, T eta, T* deltas_out) {
    const int L = n_sizes - 1;
    int64_t nact = 0;
    for (int l = 1; l <= L; ++l) nact += sizes[l];
    std::vector<T> acts(nact), deltas(nact), probs(sizes[L]);
    forward<T>(sizes, n_sizes, params, x0, acts.data(), probs.data());
    const T loss = -std::log(probs[label]);

    /* offsets of layer l's activations / deltas and parameters */
    std::vector<int64_t> aoff(L + 2, 0), poff(L + 2, 0);
    for (int l = 1; l <= L; ++l) {
        aoff[l + 1] = aoff[l] + sizes[l];
        poff[l + 1] = poff[l] + (int64_t)(sizes[l - 1] + 1) * sizes[l];
    }
    /* output delta of softmax + cross-entropy: p - onehot */
    T* dL = deltas.data() + aoff[L];
    for (int k = 0; k < sizes[L]; ++k) dL[k] = probs[k] - (k == label ? T(1) : T(0));

    /* pass 1: deltas of every hidden layer, old weights throughout */
    for (int l = L; l >= 2; --l) {
        const int nin = sizes[l - 1], nout = sizes[l];
        const T* W = params + poff[l];
        const T* d = deltas.data() + aoff[l];
        const T* xprev = acts.data() + aoff[l - 1];
        T* dprev = deltas.data() + aoff[l - 1];
#pragma omp parallel for num_threads(g_threads) if (g_threads > 1)
        for (int i = 0; i < nin; ++i) {
            T g = 0;
            for (int j = 0; j < nout; ++j) g += W[(int64_t)j * nin + i] * d[j];
            dprev[i] = g * dact_from_y<T>(xprev[i]);
        }
    }
    /* pass 2: weight updates */
    for (int l = 1; l <= L; ++l) {
        const int nin = sizes[l - 1], nout = sizes[l];
        T* W = params + poff[l];
        T* b = W + (int64_t)nin * nout;
        const T* d = deltas.data() + aoff[l];
        const T* xin = (l == 1) ? x0 : acts.data() + aoff[l - 1];
#pragma omp parallel for num_threads(g_threads) if (g_threads > 1)
        for (int j = 0; j < nout; ++j) {
            const T ed = eta * d[j];
            for (int i = 0; i < nin; ++i) W[(int64_t)j * nin + i] -= ed * xin[i];
            b[j] -= ed;
        }
    }
    if (deltas_out) std::memcpy(deltas_out, deltas.data(), sizeof(T) * nact);
    return loss;
}

template <class T>
void classify(const int32_t* sizes, int32_t n_sizes, const T* params, const T* samples, int64_t n, int32_t* out) {
    const int L = n_sizes - 1;
    int64_t nact = 0;
    for (int l = 1; l <= L; ++l) nact += sizes[l];
    std::vector<T> acts(nact), probs(sizes[L]);
    for (int64_t s = 0; s < n; ++s) {
        forward<T>(sizes, n_sizes, params, samples + s * sizes[0], acts.data(), probs.data());
        const T* a = acts.data() + (nact - sizes[L]);      /* argmax over the logits, lowest index wins ties */
        int best = 0;
        for (int k = 1; k < sizes[L]; ++k) if (a[k] > a[best]) best = k;
        out[s] = best;
    }
}

/* Output-layer pre-activations (logits) of n samples, sample by sample through
 * forward(); the samples are independent, so they may be dealt to threads (each
 * sample is then propagated by one thread, sums in the same order as ever). */
template <class T>
void logits_batch(const int32_t* sizes, int32_t n_sizes, const T* params, const T* samples, int64_t n, T* out) {
    const int L = n_sizes - 1;
    int64_t nact = 0;
    for (int l = 1; l <= L; ++l) nact += sizes[l];
    const int threads = g_threads;
#pragma omp parallel num_threads(threads) if (threads > 1)
    {
        std::vector<T> acts(nact), probs(sizes[L]);
#pragma omp for schedule(dynamic, 4)
        for (int64_t s = 0; s < n; ++s) {
            forward<T>(sizes, n_sizes, params, samples + s * sizes[0], acts.data(), probs.data());
            for (int k = 0; k < sizes[L]; ++k) out[s * sizes[L] + k] = acts[nact - sizes[L] + k];
        }
    }
}

/* ------------------------------------------------------------------------
 * Deformation (section "Deforming images ...", appendix "Deformations").
 * ---------------------------------------------------------------------- */

/* 1-D Gaussian taps t = -(k-1)/2 .. (k-1)/2, exp(-t^2 / (2 sigma^2)), scaled to sum 1.
 * sigma == 0 means no smoothing: a unit impulse. */
template <class T>
void gauss_taps(T sigma, int ktaps, T* taps) {
    const int R = (ktaps - 1) / 2;
    T s = 0;
    for (int t = -R; t <= R; ++t) {
        T v = (sigma > 0) ? std::exp(-(T)(t * t) / (2 * sigma * sigma)) : (t == 0 ? T(1) : T(0));
        taps[t + R] = v;
        s += v;
    }
    for (int i = 0; i < ktaps; ++i) taps[i] = taps[i] / s;
}

/* Smooth an H x W field with the separable Gaussian: along rows first (index c),
 * then along columns (index r); the field is zero outside; result times alpha. */
template <class T>
void smooth_field(const T* field, int H, int W, T sigma, int ktaps, T alpha, T* out) {
    const int R = (ktaps - 1) / 2;
    std::vector<T> taps(ktaps), tmp((size_t)H * W);
    gauss_taps<T>(sigma, ktaps, taps.data());
    for (int r = 0; r < H; ++r)
        for (int c = 0; c < W; ++c) {
            T s = 0;
            for (int t = -R; t <= R; ++t) {
                const int cc = c + t;
                if (cc >= 0 && cc < W) s += taps[t + R] * field[r * W + cc];
            }
            tmp[r * W + c] = s;
        }
    for (int r = 0; r < H; ++r)
        for (int c = 0; c < W; ++c) {
            T s = 0;
            for (int t = -R; t <= R; ++t) {
                const int rr = r + t;
                if (rr >= 0 && rr < H) s += taps[t + R] * tmp[rr * W + c];
            }
            out[r * W + c] = alpha * s;
        }
}

/* Random numbers of image `index`: counter 0: rotation, 1: x scale, 2: y scale,
 * 3 .. 3+HW-1: x displacement field row-major, then HW values of the y field. */
void draw_image_randoms(uint64_t seed, uint64_t index, int HW, float* s3, float* Dx, float* Dy) {
    const uint64_t key = stream_key(seed, index);
    for (int i = 0; i < 3; ++i) s3[i] = sym_unit(draw(key, i));
    for (int i = 0; i < HW; ++i) Dx[i] = sym_unit(draw(key, 3 + (uint64_t)i));
    for (int i = 0; i < HW; ++i) Dy[i] = sym_unit(draw(key, 3 + (uint64_t)HW + i));
}

/* Per-image scalars are formed in double and then rounded to T:
 * angle = beta * s0 degrees, scales 1 + (gamma/100) * s1, 1 + (gamma/100) * s2. */
template <class T>
void affine_scalars(float beta_deg, float gamma_pct, const float* s3, T* cs, T* sn, T* sx, T* sy) {
    const double th = (double)beta_deg * (double)s3[0] * (3.14159265358979323846 / 180.0);
    *cs = (T)std::cos(th);
    *sn = (T)std::sin(th);
    *sx = (T)(1.0 + ((double)gamma_pct / 100.0) * (double)s3[1]);
    *sy = (T)(1.0 + ((double)gamma_pct / 100.0) * (double)s3[2]);
}

/* The linear part of the inverse map, applied to (u, v) = output pixel minus centre:
 *   X' = p u + q v,  Y' = r u + t v   (then scaled by sx, sy).
 * Rotation by the angle: (p, q, r, t) = (cos, -sin, sin, cos).
 * Horizontal shear (section "Deforming images ..."): the tangent of the angle is the ratio of
 * horizontal displacement to height, so a row v above or below the centre moves by tan * v:
 * (p, q, r, t) = (1, tan, 0, 1).  Formed in double from the same angle, rounded to T. */
template <class T>
void linear_part(int shear, float beta_deg, const float* s3, T* pqrt) {
    const double th = (double)beta_deg * (double)s3[0] * (3.14159265358979323846 / 180.0);
    if (shear) {
        pqrt[0] = (T)1; pqrt[1] = (T)std::tan(th); pqrt[2] = (T)0; pqrt[3] = (T)1;
    } else {
        pqrt[0] = (T)std::cos(th); pqrt[1] = (T)(-std::sin(th)); pqrt[2] = (T)std::sin(th); pqrt[3] = (T)std::cos(th);
    }
}

/* Inverse-map resampling: output pixel (r,c) takes the bilinear sample of the
 * source image at
 *   X = sx (p u + q v) + c0x + dx[r][c],   u = c - c0x, c0x = (W-1)/2
 *   Y = sy (r u + t v) + c0y + dy[r][c],   v = r - c0y, c0y = (H-1)/2
 * every one of the four taps being 0 (background) when it lies outside the
 * image.  The result is mapped to intensity/127.5 - 1 (section "Data"). */
template <class T>
void resample_lin(const uint8_t* img, int H, int W, const T* pqrt, T sx, T sy, const T* dx, const T* dy, T* out) {
    const T c0x = (T)(W - 1) / 2, c0y = (T)(H - 1) / 2;
    for (int r = 0; r < H; ++r)
        for (int c = 0; c < W; ++c) {
            const T u = (T)c - c0x, v = (T)r - c0y;
            const T X = sx * (pqrt[0] * u + pqrt[1] * v) + c0x + dx[r * W + c];
            const T Y = sy * (pqrt[2] * u + pqrt[3] * v) + c0y + dy[r * W + c];
            const T xf = std::floor(X), yf = std::floor(Y);
            const T fx = X - xf, fy = Y - yf;
            T p00 = 0, p01 = 0, p10 = 0, p11 = 0;
            /* guard the float -> int conversion for far-away coordinates */
            if (xf >= -1 && xf <= (T)W && yf >= -1 && yf <= (T)H) {
                const int x0 = (int)xf, y0 = (int)yf;
                auto P = [&](int y, int x) -> T {
                    return (x >= 0 && x < W && y >= 0 && y < H) ? (T)img[y * W + x] : T(0);
                };
                p00 = P(y0, x0); p01 = P(y0, x0 + 1); p10 = P(y0 + 1, x0); p11 = P(y0 + 1, x0 + 1);
            }
            const T val = (1 - fy) * ((1 - fx) * p00 + fx * p01) + fy * ((1 - fx) * p10 + fx * p11);
            out[r * W + c] = val / (T)127.5 - 1;
        }
}

/* Rotation given as cosine and sine. */
template <class T>
void resample(const uint8_t* img, int H, int W, T cs, T sn, T sx, T sy, const T* dx, const T* dy, T* out) {
    const T pqrt[4] = {cs, -sn, sn, cs};
    resample_lin<T>(img, H, W, pqrt, sx, sy, dx, dy, out);
}

template <class T>
void deform_one(float sigma, float alpha, float beta_deg, float gamma_pct, int ktaps, int shear, const uint8_t* img,
                uint64_t seed, uint64_t index, T* out) {
    const int H = 28, W = 28, HW = H * W;
    float s3[3];
    std::vector<float> Dx(HW), Dy(HW);
    draw_image_randoms(seed, index, HW, s3, Dx.data(), Dy.data());
    std::vector<T> fx(HW), fy(HW), gx(HW), gy(HW);
    for (int i = 0; i < HW; ++i) { fx[i] = (T)Dx[i]; fy[i] = (T)Dy[i]; }
    smooth_field<T>(fx.data(), H, W, (T)sigma, ktaps, (T)alpha, gx.data());
    smooth_field<T>(fy.data(), H, W, (T)sigma, ktaps, (T)alpha, gy.data());
    T cs, sn, sx, sy, pqrt[4];
    affine_scalars<T>(beta_deg, gamma_pct, s3, &cs, &sn, &sx, &sy);
    linear_part<T>(shear, beta_deg, s3, pqrt);
    resample_lin<T>(img, H, W, pqrt, sx, sy, gx.data(), gy.data(), out);
}

}  // namespace

extern "C" {

void dbsn_oracle_set_threads(int32_t n) {
#ifdef _OPENMP
    g_threads = n < 1 ? 1 : n;
#else
    (void)n; g_threads = 1;
#endif
}
int32_t dbsn_oracle_get_threads(void) { return g_threads; }
int32_t dbsn_oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

int64_t dbsn_oracle_param_count(const int32_t* sizes, int32_t n_sizes) { return param_count(sizes, n_sizes); }

void dbsn_oracle_rng_raw(uint64_t seed, uint64_t stream, uint64_t first_counter, int64_t n, uint64_t* out) {
    const uint64_t key = stream_key(seed, stream);
    for (int64_t i = 0; i < n; ++i) out[i] = draw(key, first_counter + (uint64_t)i);
}
void dbsn_oracle_rng_sym(uint64_t seed, uint64_t stream, uint64_t first_counter, int64_t n, float* out) {
    const uint64_t key = stream_key(seed, stream);
    for (int64_t i = 0; i < n; ++i) out[i] = sym_unit(draw(key, first_counter + (uint64_t)i));
}

/* Weight initialisation (section "Architectures"): uniform in [-0.05, 0.05).
 * Layer l uses stream l; W_l[j][i] takes counter j*(n_{l-1}+1)+i and the bias
 * b_l[j] takes counter j*(n_{l-1}+1)+n_{l-1}; value = k * (0.05 * 2^-23) with
 * k the signed 24-bit integer of the draw (one float multiply, exact scale). */
void dbsn_oracle_init_params_f32(const int32_t* sizes, int32_t n_sizes, uint64_t seed, float* params) {
    const float scale = 0.05f / 8388608.0f;
    float* p = params;
    for (int l = 1; l < n_sizes; ++l) {
        const int nin = sizes[l - 1], nout = sizes[l];
        const uint64_t key = stream_key(seed, (uint64_t)l);
        float* W = p;
        float* b = p + (int64_t)nin * nout;
        for (int j = 0; j < nout; ++j) {
            for (int i = 0; i <= nin; ++i) {
                const uint64_t r = draw(key, (uint64_t)j * (uint64_t)(nin + 1) + (uint64_t)i);
                const int32_t k = (int32_t)(r >> 40) - (1 << 23);
                const float w = (float)k * scale;
                if (i < nin) W[(int64_t)j * nin + i] = w; else b[j] = w;
            }
        }
        p += (int64_t)(nin + 1) * nout;
    }
}

#define DBSN_ORACLE_MLP(SUF, T)                                                                                     \
    void dbsn_oracle_forward_##SUF(const int32_t* sizes, int32_t n_sizes, const T* params, const T* x0, T* acts,    \
                                   T* probs) {                                                                      \
        forward<T>(sizes, n_sizes, params, x0, acts, probs);                                                        \
    }                                                                                                               \
    T dbsn_oracle_bp_step_##SUF(const int32_t* sizes, int32_t n_sizes, T* params, const T* x0, int32_t label,       \
                                T eta, T* deltas_out) {                                                             \
        return bp_step<T>(sizes, n_sizes, params, x0, label, eta, deltas_out);                                      \
    }                                                                                                               \
    void dbsn_oracle_bp_steps_##SUF(const int32_t* sizes, int32_t n_sizes, T* params, const T* samples,             \
                                    const int32_t* labels, int64_t n, T eta, T* loss_out) {                         \
        for (int64_t s = 0; s < n; ++s) {                                                                           \
            T loss = bp_step<T>(sizes, n_sizes, params, samples + s * sizes[0], labels[s], eta, nullptr);           \
            if (loss_out) loss_out[s] = loss;                                                                       \
        }                                                                                                           \
    }                                                                                                               \
    void dbsn_oracle_classify_##SUF(const int32_t* sizes, int32_t n_sizes, const T* params, const T* samples,       \
                                    int64_t n, int32_t* out) {                                                      \
        classify<T>(sizes, n_sizes, params, samples, n, out);                                                       \
    }                                                                                                               \
    void dbsn_oracle_logits_batch_##SUF(const int32_t* sizes, int32_t n_sizes, const T* params, const T* samples,   \
                                        int64_t n, T* out) {                                                        \
        logits_batch<T>(sizes, n_sizes, params, samples, n, out);                                                   \
    }                                                                                                               \
    T dbsn_oracle_act_##SUF(T a) { return act<T>(a); }                                                              \
    T dbsn_oracle_dact_from_y_##SUF(T y) { return dact_from_y<T>(y); }                                              \
    void dbsn_oracle_gauss_taps_##SUF(T sigma, int32_t ktaps, T* taps) { gauss_taps<T>(sigma, ktaps, taps); }      \
    void dbsn_oracle_smooth_field_##SUF(const T* field, int32_t H, int32_t W, T sigma, int32_t ktaps, T alpha,      \
                                        T* out) {                                                                   \
        smooth_field<T>(field, H, W, sigma, ktaps, alpha, out);                                                     \
    }                                                                                                               \
    void dbsn_oracle_affine_scalars_##SUF(float beta_deg, float gamma_pct, const float* s3, T* out4) {              \
        affine_scalars<T>(beta_deg, gamma_pct, s3, out4, out4 + 1, out4 + 2, out4 + 3);                             \
    }                                                                                                               \
    void dbsn_oracle_resample_##SUF(const uint8_t* img, int32_t H, int32_t W, T cs, T sn, T sx, T sy, const T* dx,  \
                                    const T* dy, T* out) {                                                          \
        resample<T>(img, H, W, cs, sn, sx, sy, dx, dy, out);                                                        \
    }                                                                                                               \
    void dbsn_oracle_linear_part_##SUF(int32_t shear, float beta_deg, const float* s3, T* pqrt) {                   \
        linear_part<T>(shear, beta_deg, s3, pqrt);                                                                  \
    }                                                                                                               \
    void dbsn_oracle_resample_lin_##SUF(const uint8_t* img, int32_t H, int32_t W, const T* pqrt, T sx, T sy,        \
                                        const T* dx, const T* dy, T* out) {                                         \
        resample_lin<T>(img, H, W, pqrt, sx, sy, dx, dy, out);                                                      \
    }                                                                                                               \
    /* beta_each: one angle bound per image (degrees), or NULL for beta_deg everywhere */                          \
    void dbsn_oracle_deform_batch_##SUF(float sigma, float alpha, float beta_deg, float gamma_pct, int32_t ktaps,   \
                                        int32_t shear, const float* beta_each, const uint8_t* src, int64_t n,       \
                                        uint64_t seed, uint64_t first_index, T* dst) {                              \
        _Pragma("omp parallel for num_threads(g_threads) if (g_threads > 1)")                                       \
        for (int64_t k = 0; k < n; ++k)                                                                             \
            deform_one<T>(sigma, alpha, beta_each ? beta_each[k] : beta_deg, gamma_pct, ktaps, shear,               \
                          src + k * 784, seed, first_index + (uint64_t)k, dst + k * 784);                           \
    }

DBSN_ORACLE_MLP(f32, float)
DBSN_ORACLE_MLP(f64, double)

void dbsn_oracle_draw_image_randoms(uint64_t seed, uint64_t index, int32_t HW, float* s3, float* Dx, float* Dy) {
    draw_image_randoms(seed, index, HW, s3, Dx, Dy);
}

}  // extern "C"
