// AdamW factor of the weight-divergence estimate (SNIP Sec. 4.3.2 "Impact on Weight Divergence").
// With m = beta1 m' + (1 - beta1) g and v = beta2 v' + (1 - beta2) g^2, the update direction
// h(g) = m / (sqrt(v) + eps) has the element-wise derivative
//     (1 - beta1) / (sqrt(v) + eps)  -  (1 - beta2) m g / (sqrt(v) (sqrt(v) + eps)^2),
// and Step 1 of the method collects its Frobenius norm.  One streaming pass over m, v (fp32) and
// g (fp32 or bf16): 12 or 10 bytes per element read, nothing written but one partial per wave, so
// the kernel is bound by HBM bandwidth (about 25 VALU slots per element, far below the ~70 a CU can
// spend per element at that rate).  fp32 arithmetic with correctly rounded square root and division;
// sums per lane and wave in fp32, across waves in double in a fixed order.
#include "snip_internal.h"

namespace snip {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float sens_term(float m, float v, float g, float c1, float c2, float eps)
{
    const float root = __fsqrt_rn(v);
    const float d = root + eps;
    const float first = __fdiv_rn(c1, d);
    // v == 0: AdamW has m = g = 0 there and the second part is taken as zero (the expression is 0/0)
    const float second = v > 0.f ? __fdiv_rn(c2 * m * g, root * d * d) : 0.f;
    const float t = first - second;
    return t * t;
}

template <bool G_BF16>
__global__ __launch_bounds__(256) void adamw_sens_kernel(const float* __restrict__ m, const float* __restrict__ v,
                                                         const void* __restrict__ g, int64_t n, float c1, float c2,
                                                         float eps, float* __restrict__ partials)
{
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t nthreads = (int64_t)gridDim.x * 256;
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n4 = n / 4;
    float acc = 0.f;
    for (int64_t q = tid; q < n4; q += nthreads) {
        // streaming (non-temporal) loads: nothing is read twice and the three arrays exceed every cache
        const v4f mm = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(m) + q);
        const v4f vv = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(v) + q);
        v4f gg;
        if (G_BF16) {
            const v2u w = __builtin_nontemporal_load(reinterpret_cast<const v2u*>(g) + q);
            gg = v4f{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xFFFF0000u),
                     __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xFFFF0000u)};
        } else {
            gg = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(g) + q);
        }
        acc += sens_term(mm.x, vv.x, gg.x, c1, c2, eps);
        acc += sens_term(mm.y, vv.y, gg.y, c1, c2, eps);
        acc += sens_term(mm.z, vv.z, gg.z, c1, c2, eps);
        acc += sens_term(mm.w, vv.w, gg.w, c1, c2, eps);
    }
    // the last n % 4 elements
    const int64_t i = n4 * 4 + tid;
    if (i < n) {
        const float gi = G_BF16 ? __uint_as_float((unsigned)reinterpret_cast<const uint16_t*>(g)[i] << 16)
                                : reinterpret_cast<const float*>(g)[i];
        acc += sens_term(m[i], v[i], gi, c1, c2, eps);
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) partials[wave] = acc;
}

}  // namespace

hipError_t launch_adamw_sensitivity(const AdamwArgs& a, hipStream_t s)
{
    float* partials = (float*)a.workspace;
    if (a.n > 0) {
        const float c1 = 1.0f - a.beta1, c2 = 1.0f - a.beta2;
        if (a.g_bf16)
            hipLaunchKernelGGL(adamw_sens_kernel<true>, dim3(kStreamBlocks), dim3(256), 0, s, a.m, a.v, a.g, a.n, c1, c2, a.eps, partials);
        else
            hipLaunchKernelGGL(adamw_sens_kernel<false>, dim3(kStreamBlocks), dim3(256), 0, s, a.m, a.v, a.g, a.n, c1, c2, a.eps, partials);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return launch_sum_partials(partials, a.n > 0 ? kStreamWaves : 0, a.out, s);
}

}  // namespace snip
