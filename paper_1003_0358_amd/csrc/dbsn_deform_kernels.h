// Deformation kernel of libdbsn for gfx950 (section "Deforming images to get more training
// instances", appendix "Deformations").
//
// One workgroup of 256 threads deforms one 28x28 image entirely in LDS: it draws the two random
// displacement fields, smooths them with the separable Gaussian (rows, then columns, the field
// being zero outside the image), scales them by alpha, adds the rotated (or horizontally sheared)
// and scaled pixel grid and takes the bilinear sample of the source image.  The paper ran only the (full 2-D, 441-tap)
// convolution on its GPU and everything else on the CPU; here nothing leaves the chip between the
// uint8 source (784 B read) and the float result (3136 B written).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dbsn_rng.h"

namespace dbsn {

constexpr int kSide = 28;
constexpr int kPix = kSide * kSide;
constexpr int kDeformThreads = 256;
constexpr int kMaxTaps = 63;

struct DeformArgs {
    float taps[kMaxTaps + 1];  // 1-D Gaussian, sums to 1, taps[R] is the centre
    int ktaps;
    float alpha, beta_deg, gamma_pct;
    int shear;                 // 0: rotation by the angle, 1: horizontal shear with tan(angle) = displacement / height
    const float* beta_each;    // per-image bound of the angle in degrees, or null
    const int* labels;         // or: per-image class labels (null: beta_deg everywhere); an image whose class has its
    uint64_t similar_mask;     //   bit set in similar_mask (bit c = class c < 64) takes beta_similar, any other beta_deg
    float beta_similar;
    uint64_t seed, first_index;
    long long n;
};

// Per-image scalars of image k (one thread): the linear part p, q, r, t of the inverse map
// (X' = p u + q v, Y' = r u + t v) and the two scale factors, formed in double from the first three
// draws of the image's stream and rounded once to float.  The bound of the angle is the image's own
// (beta_each), or follows its class label (section "Deforming images ...": look-alike classes are
// rotated or sheared less), or is beta_deg.
__device__ inline void image_affine(const DeformArgs& a, uint64_t key, long long k, float* aff) {
    const double u0 = (double)rng_unit(rng_draw(key, 0));
    const double u1 = (double)rng_unit(rng_draw(key, 1));
    const double u2 = (double)rng_unit(rng_draw(key, 2));
    double beta = (double)a.beta_deg;
    if (a.beta_each) {
        beta = (double)a.beta_each[k];
    } else if (a.labels) {
        const int c = a.labels[k];
        if (c >= 0 && c < 64 && ((a.similar_mask >> c) & 1ull)) beta = (double)a.beta_similar;
    }
    const double th = beta * u0 * (3.14159265358979323846 / 180.0);
    if (a.shear) {
        aff[0] = 1.0f; aff[1] = (float)tan(th); aff[2] = 0.0f; aff[3] = 1.0f;
    } else {
        aff[0] = (float)cos(th); aff[1] = (float)(-sin(th)); aff[2] = (float)sin(th); aff[3] = (float)cos(th);
    }
    aff[4] = (float)(1.0 + ((double)a.gamma_pct / 100.0) * u1);
    aff[5] = (float)(1.0 + ((double)a.gamma_pct / 100.0) * u2);
}

__global__ __launch_bounds__(kDeformThreads) void k_deform(DeformArgs a, const uint8_t* __restrict__ src,
                                                            float* __restrict__ dst) {
    __shared__ float img[kPix];
    __shared__ float fx[kPix], fy[kPix];   // raw fields, later reused for nothing else
    __shared__ float tx[kPix], ty[kPix];   // after the row pass
    __shared__ float aff[6];               // linear part p, q, r, t (X' = p u + q v, Y' = r u + t v), then sx, sy
    const int R = (a.ktaps - 1) / 2;

    for (long long k = blockIdx.x; k < a.n; k += gridDim.x) {
        const uint64_t key = rng_key(a.seed, a.first_index + (uint64_t)k);
        const uint8_t* s = src + k * kPix;
        for (int i = threadIdx.x; i < kPix; i += kDeformThreads) {
            img[i] = (float)s[i];
            fx[i] = rng_unit(rng_draw(key, 3ull + (uint64_t)i));
            fy[i] = rng_unit(rng_draw(key, 3ull + (uint64_t)kPix + (uint64_t)i));
        }
        if (threadIdx.x == 0) image_affine(a, key, k, aff);
        __syncthreads();
        // row pass: along c
        for (int i = threadIdx.x; i < kPix; i += kDeformThreads) {
            const int r = i / kSide, c = i - r * kSide;
            float sx = 0.0f, sy = 0.0f;
            for (int t = -R; t <= R; ++t) {
                const int cc = c + t;
                if (cc >= 0 && cc < kSide) {
                    const float w = a.taps[t + R];
                    sx = fmaf(w, fx[r * kSide + cc], sx);
                    sy = fmaf(w, fy[r * kSide + cc], sy);
                }
            }
            tx[i] = sx;
            ty[i] = sy;
        }
        __syncthreads();
        const float lp = aff[0], lq = aff[1], lr = aff[2], lt = aff[3], scx = aff[4], scy = aff[5];
        const float c0 = 0.5f * (float)(kSide - 1);
        float* out = dst + k * kPix;
        for (int i = threadIdx.x; i < kPix; i += kDeformThreads) {
            const int r = i / kSide, c = i - r * kSide;
            // column pass: along r
            float gx = 0.0f, gy = 0.0f;
            for (int t = -R; t <= R; ++t) {
                const int rr = r + t;
                if (rr >= 0 && rr < kSide) {
                    const float w = a.taps[t + R];
                    gx = fmaf(w, tx[rr * kSide + c], gx);
                    gy = fmaf(w, ty[rr * kSide + c], gy);
                }
            }
            const float u = (float)c - c0, v = (float)r - c0;
            // X = sx (p u + q v) + c0 + alpha * smoothed dx;  Y = sy (r u + t v) + c0 + alpha * smoothed dy
            const float X = fmaf(a.alpha, gx, fmaf(scx, fmaf(lp, u, lq * v), c0));
            const float Y = fmaf(a.alpha, gy, fmaf(scy, fmaf(lr, u, lt * v), c0));
            const float xf = floorf(X), yf = floorf(Y);
            const float wx = X - xf, wy = Y - yf;
            float p00 = 0.f, p01 = 0.f, p10 = 0.f, p11 = 0.f;
            if (xf >= -1.0f && xf <= (float)kSide && yf >= -1.0f && yf <= (float)kSide) {
                const int x0 = (int)xf, y0 = (int)yf;
                const bool xa = (x0 >= 0 && x0 < kSide), xb = (x0 + 1 >= 0 && x0 + 1 < kSide);
                const bool ya = (y0 >= 0 && y0 < kSide), yb = (y0 + 1 >= 0 && y0 + 1 < kSide);
                if (ya && xa) p00 = img[y0 * kSide + x0];
                if (ya && xb) p01 = img[y0 * kSide + x0 + 1];
                if (yb && xa) p10 = img[(y0 + 1) * kSide + x0];
                if (yb && xb) p11 = img[(y0 + 1) * kSide + x0 + 1];
            }
            const float top = (1.0f - wx) * p00 + wx * p01;
            const float bot = (1.0f - wx) * p10 + wx * p11;
            const float val = (1.0f - wy) * top + wy * bot;
            out[i] = val / 127.5f - 1.0f;   // section "Data": intensity/127.5 - 1
        }
        __syncthreads();   // LDS is reused by the next image of this workgroup
    }
}

// The same deformation with the number of taps known at compile time, for the 21 taps the paper
// uses.  k_deform above spends most of its instructions around the convolutions (per tap and
// field: a bounds test, an index, an LDS read, a tap fetch for one multiply-add).  Here the fields
// live in LDS lines padded with zeros on both sides (no bounds test: a tap outside the image adds
// an exact zero, where k_deform adds nothing, so the sums are the same numbers), a thread computes
// four neighbouring outputs of both fields from one window of 4 + 2R values read as float4 (one
// LDS read per 14 multiply-adds), the taps sit in scalar registers, and the row pass writes its
// result transposed, so that the column pass is the same walk along a line; it puts its result
// back into the field lines, and the resampling then takes a pixel per thread like k_deform.
// Every sum runs over the taps in the order of k_deform: the two kernels agree bit for bit.
constexpr int kPadLine = 52;   // floats per padded line: 13 float4, and 52 * c mod 64 visits 16 bank groups

template <int KT>
__global__ __launch_bounds__(kDeformThreads, 4) void k_deform_taps(DeformArgs a, const uint8_t* __restrict__ src,
                                                                 float* __restrict__ dst) {
    constexpr int R = (KT - 1) / 2;
    constexpr int kWin = 4 + 2 * R;                 // values a run of four outputs needs
    static_assert(KT == 2 * R + 1 && kWin % 4 == 0 && kSide + 2 * R <= kPadLine, "window of whole float4 inside a line");
    constexpr int kRuns = kSide / 4;                // runs of four outputs per line
    constexpr int kItems = kSide * kRuns;           // (line, run) pairs: 196 of the 256 threads work
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ float img[kPix];
    __shared__ __attribute__((aligned(16))) float fld[2][kSide][kPadLine];   // raw fields: line r, pixel c at [R + c]
    __shared__ __attribute__((aligned(16))) float row[2][kSide][kPadLine];   // after the row pass, transposed: line c, pixel r at [R + r]
    __shared__ float aff[6];               // linear part p, q, r, t (X' = p u + q v, Y' = r u + t v), then sx, sy
    for (int i = threadIdx.x; i < 2 * kSide * kPadLine; i += kDeformThreads) {
        (&fld[0][0][0])[i] = 0.0f;   // the padding stays zero from here on
        (&row[0][0][0])[i] = 0.0f;
    }
    float w[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t) w[t] = a.taps[t];
    const int line = threadIdx.x / kRuns, run = threadIdx.x - line * kRuns;   // row pass: image row, run of columns
    const int crun = threadIdx.x / kSide, ccol = threadIdx.x - crun * kSide;   // column pass: run of rows, image column
    __syncthreads();

    for (long long k = blockIdx.x; k < a.n; k += gridDim.x) {
        const uint64_t key = rng_key(a.seed, a.first_index + (uint64_t)k);
        const uint8_t* s = src + k * kPix;
        for (int i = threadIdx.x; i < kPix; i += kDeformThreads) {
            const int r = i / kSide, c = i - r * kSide;
            img[i] = (float)s[i];
            fld[0][r][R + c] = rng_unit(rng_draw(key, 3ull + (uint64_t)i));
            fld[1][r][R + c] = rng_unit(rng_draw(key, 3ull + (uint64_t)kPix + (uint64_t)i));
        }
        if (threadIdx.x == 0) image_affine(a, key, k, aff);
        __syncthreads();
        // row pass: outputs (line, 4 run .. 4 run + 3) of both fields; the window starts at padded index 4 run
        if (threadIdx.x < kItems) {
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                float in[kWin];
#pragma unroll
                for (int q = 0; q < kWin / 4; ++q) {
                    const f4 v = *reinterpret_cast<const f4*>(&fld[f][line][4 * run + 4 * q]);
                    in[4 * q] = v[0]; in[4 * q + 1] = v[1]; in[4 * q + 2] = v[2]; in[4 * q + 3] = v[3];
                }
#pragma unroll
                for (int o = 0; o < 4; ++o) {
                    float sum = 0.0f;
#pragma unroll
                    for (int t = 0; t < KT; ++t) sum = fmaf(w[t], in[o + t], sum);
                    row[f][4 * run + o][R + line] = sum;
                }
            }
        }
        __syncthreads();
        const float lp = aff[0], lq = aff[1], lr = aff[2], lt = aff[3], scx = aff[4], scy = aff[5];
        const float c0 = 0.5f * (float)(kSide - 1);
        float* out = dst + k * kPix;
        // column pass: pixels (4 crun .. 4 crun + 3, ccol) of both fields, back into the field lines
        // (the raw fields are spent)
        if (threadIdx.x < kItems) {
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                float in[kWin];
#pragma unroll
                for (int q = 0; q < kWin / 4; ++q) {
                    const f4 v = *reinterpret_cast<const f4*>(&row[f][ccol][4 * crun + 4 * q]);
                    in[4 * q] = v[0]; in[4 * q + 1] = v[1]; in[4 * q + 2] = v[2]; in[4 * q + 3] = v[3];
                }
#pragma unroll
                for (int o = 0; o < 4; ++o) {
                    float sum = 0.0f;
#pragma unroll
                    for (int t = 0; t < KT; ++t) sum = fmaf(w[t], in[o + t], sum);
                    fld[f][4 * crun + o][R + ccol] = sum;
                }
            }
        }
        __syncthreads();
        // resampling, a pixel per thread and round
        for (int i = threadIdx.x; i < kPix; i += kDeformThreads) {
            const int r = i / kSide, c = i - r * kSide;
            const float gx = fld[0][r][R + c], gy = fld[1][r][R + c];
            const float u = (float)c - c0, v = (float)r - c0;
            // X = sx (p u + q v) + c0 + alpha * smoothed dx;  Y = sy (r u + t v) + c0 + alpha * smoothed dy
            const float X = fmaf(a.alpha, gx, fmaf(scx, fmaf(lp, u, lq * v), c0));
            const float Y = fmaf(a.alpha, gy, fmaf(scy, fmaf(lr, u, lt * v), c0));
            const float xf = floorf(X), yf = floorf(Y);
            const float wx = X - xf, wy = Y - yf;
            float p00 = 0.f, p01 = 0.f, p10 = 0.f, p11 = 0.f;
            if (xf >= -1.0f && xf <= (float)kSide && yf >= -1.0f && yf <= (float)kSide) {
                const int x0 = (int)xf, y0 = (int)yf;
                const bool xa = (x0 >= 0 && x0 < kSide), xb = (x0 + 1 >= 0 && x0 + 1 < kSide);
                const bool ya = (y0 >= 0 && y0 < kSide), yb = (y0 + 1 >= 0 && y0 + 1 < kSide);
                if (ya && xa) p00 = img[y0 * kSide + x0];
                if (ya && xb) p01 = img[y0 * kSide + x0 + 1];
                if (yb && xa) p10 = img[(y0 + 1) * kSide + x0];
                if (yb && xb) p11 = img[(y0 + 1) * kSide + x0 + 1];
            }
            const float top = (1.0f - wx) * p00 + wx * p01;
            const float bot = (1.0f - wx) * p10 + wx * p11;
            const float val = (1.0f - wy) * top + wy * bot;
            out[i] = val / 127.5f - 1.0f;   // section "Data": intensity/127.5 - 1
        }
        __syncthreads();   // LDS is reused by the next image of this workgroup
    }
}

}  // namespace dbsn
