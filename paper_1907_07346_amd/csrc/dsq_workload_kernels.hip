// Bit-reproducible synthetic gradients on the GPU (harness aid, not part of DeepSqueeze): the device twin
// of paper_1907_07346_amd/detgen.py.  Every value is a pure function of (seed, tag, t, worker, column):
// Philox4x32-10 words -> uniforms (word + 0.5) 2^-32 -> Box-Muller in double, with ln, sin and cos evaluated by
// the fixed polynomials below in plain IEEE double operations (the file is compiled with contraction off and
// uses no fused multiply-add), in the same order as the numpy code, so host and device agree bit for bit.
// Long free runs can then draw their gradients where the state lives.

#include "dsq_internal.h"

namespace dsq {
namespace {

constexpr uint32_t kTagCentre = 0x43454E54u, kTagNoise = 0x47524144u;     // 'CENT', 'GRAD'
constexpr double kLn2 = 0x1.62e42fefa39efp-1, kHalfPi = 0x1.921fb54442d18p+0, kSqrtHalf = 0x1.6a09e667f3bcdp-1;
constexpr int kLogTerms = 13, kTrigTerms = 14;
// 1/(2k+1); (-1)^k/(2k+1)!; (-1)^k/(2k)!  -- each rounded once to double
__device__ const double kLogCoef[13] = {
    0x1.0000000000000p+0, 0x1.5555555555555p-2, 0x1.999999999999ap-3,
    0x1.2492492492492p-3, 0x1.c71c71c71c71cp-4, 0x1.745d1745d1746p-4,
    0x1.3b13b13b13b14p-4, 0x1.1111111111111p-4, 0x1.e1e1e1e1e1e1ep-5,
    0x1.af286bca1af28p-5, 0x1.8618618618618p-5, 0x1.642c8590b2164p-5,
    0x1.47ae147ae147bp-5};
__device__ const double kSinCoef[14] = {
    0x1.0000000000000p+0, -0x1.5555555555555p-3, 0x1.1111111111111p-7,
    -0x1.a01a01a01a01ap-13, 0x1.71de3a556c734p-19, -0x1.ae64567f544e4p-26,
    0x1.6124613a86d09p-33, -0x1.ae7f3e733b81fp-41, 0x1.952c77030ad4ap-49,
    -0x1.2f49b46814157p-57, 0x1.71b8ef6dcf572p-66, -0x1.761b41316381ap-75,
    0x1.3f3ccdd165fa9p-84, -0x1.d1ab1c2dccea3p-94};
__device__ const double kCosCoef[14] = {
    0x1.0000000000000p+0, -0x1.0000000000000p-1, 0x1.5555555555555p-5,
    -0x1.6c16c16c16c17p-10, 0x1.a01a01a01a01ap-16, -0x1.27e4fb7789f5cp-22,
    0x1.1eed8eff8d898p-29, -0x1.93974a8c07c9dp-37, 0x1.ae7f3e733b81fp-45,
    -0x1.6827863b97d97p-53, 0x1.e542ba4020225p-62, -0x1.0ce396db7f853p-70,
    0x1.f2cf01972f578p-80, -0x1.88e85fc6a4e5ap-89};

__device__ __forceinline__ void philox(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// ln u, u in (0, 1] and normal: u = f 2^e with f in [sqrt(1/2), sqrt 2); ln f = 2 atanh((f - 1) / (f + 1))
__device__ __forceinline__ double det_log(double u) {
    const long long bits = __double_as_longlong(u);
    int e = (int)((bits >> 52) & 0x7FF) - 1022;
    double f = __longlong_as_double((bits & 0x800FFFFFFFFFFFFFll) | 0x3FE0000000000000ll);     // [0.5, 1)
    if (f < kSqrtHalf) { f = f * 2.0; e -= 1; }
    const double s = (f - 1.0) / (f + 1.0);
    const double z = s * s;
    double p = kLogCoef[kLogTerms - 1];
#pragma unroll
    for (int k = kLogTerms - 2; k >= 0; --k) p = p * z + kLogCoef[k];
    return (double)e * kLn2 + (2.0 * s) * p;
}

// (cos 2 pi u, sin 2 pi u), u in [0, 1): quadrant from 4u, Taylor polynomials on [0, pi/2)
__device__ __forceinline__ void det_sincos_2pi(double u, double& c_out, double& s_out) {
    const double a = 4.0 * u;
    const double q = floor(a);
    const double phi = (a - q) * kHalfPi;
    const double z = phi * phi;
    double ps = kSinCoef[kTrigTerms - 1], pc = kCosCoef[kTrigTerms - 1];
#pragma unroll
    for (int k = kTrigTerms - 2; k >= 0; --k) {
        ps = ps * z + kSinCoef[k];
        pc = pc * z + kCosCoef[k];
    }
    const double s = phi * ps, c = pc;
    const int qi = (int)q;
    c_out = qi == 0 ? c : qi == 1 ? -s : qi == 2 ? -c : s;
    s_out = qi == 0 ? s : qi == 1 ? c : qi == 2 ? -s : -c;
}

__device__ __forceinline__ void box_muller(uint32_t wa, uint32_t wb, double& z0, double& z1) {
    const double u1 = ((double)wa + 0.5) * 0x1p-32;
    const double u2 = ((double)wb + 0.5) * 0x1p-32;
    const double r = sqrt(-2.0 * det_log(u1));
    double c, s;
    det_sincos_2pi(u2, c, s);
    z0 = r * c;
    z1 = r * s;
}

__device__ __forceinline__ void normals4(uint64_t seed, uint32_t tag, uint64_t t, uint32_t row, uint32_t counter, double (&z)[4]) {
    uint32_t w[4];
    philox(counter, row, (uint32_t)t, tag, (uint32_t)seed, (uint32_t)(seed >> 32), w);
    box_muller(w[0], w[1], z[0], z[1]);
    box_muller(w[2], w[3], z[2], z[3]);
}

// One thread per four columns.
__global__ void __launch_bounds__(256) workload_gradient_kernel(ds_workload w, uint64_t t, const float* __restrict__ x, uint64_t x_ld,
                                                                float* __restrict__ g, uint64_t g_ld) {
    const uint32_t row = blockIdx.y;
    const uint64_t c = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t j = 4 * c;
    if (j >= g_ld) return;
    float out[4] = {0.f, 0.f, 0.f, 0.f};                       // columns N .. g_ld-1 are written as zeros
    if (j < w.N) {
        if (w.kind == DS_GRAD_NORMAL) {
            double z[4];
            normals4(w.seed, kTagNoise, t, row, (uint32_t)c, z);
            const double sc = (double)w.scale;
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = (float)(sc * z[e]);
        } else if (w.kind == DS_GRAD_STUDENT_T3) {
            const double sc = (double)w.scale;
            for (int e = 0; e < 4 && j + e < w.N; ++e) {
                double z[4];
                normals4(w.seed, kTagNoise, t, row, (uint32_t)(j + e), z);
                out[e] = (float)(sc * z[0] / sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0));
            }
        } else {                                               // DS_GRAD_QUADRATIC: (x - c) + scale xi, in fp32
            double zc[4], zx[4];
            normals4(w.seed, kTagCentre, 0, row, (uint32_t)c, zc);
            normals4(w.seed, kTagNoise, t, row, (uint32_t)c, zx);
            for (int e = 0; e < 4 && j + e < w.N; ++e) {
                const float d = x[(uint64_t)row * x_ld + j + e] - (float)zc[e];
                const float p = w.scale * (float)zx[e];
                out[e] = d + p;
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j + e >= w.N) out[e] = 0.f;
    }
    float* dst = g + (uint64_t)row * g_ld + j;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (j + e < g_ld) dst[e] = out[e];
}

}  // namespace

ds_status launch_workload_gradient(const ds_workload& w, uint64_t t, const float* x, uint64_t x_ld, float* g, uint64_t g_ld,
                                   hipStream_t stream) {
    const uint64_t quads = (g_ld + 3) / 4;
    hipLaunchKernelGGL(workload_gradient_kernel, dim3((unsigned)((quads + 255) / 256), w.n), dim3(256), 0, stream, w, t, x, x_ld, g, g_ld);
    return hipGetLastError() == hipSuccess ? DS_OK : DS_EHIP;
}

}  // namespace dsq
