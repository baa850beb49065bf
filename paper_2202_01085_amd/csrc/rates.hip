// f3m_rates: instruction and copy rates of the device this runs on, the yardsticks that the kernel figures of
// the library are read against (the published peaks assume packed FP32 and say nothing about v_exp_f32).
// A stand-alone program, built beside the library by paper_2202_01085_amd/build.py; prints one JSON object.
//   fma        v_fma_f32, eight independent chains per lane, 8 wavefronts per SIMD
//   exp2       v_exp_f32, likewise
//   pair       the near field's per-pair work after the Gram product: one v_exp_f32 and one v_fma_f32
//   diff_pair  the exact product's per-pair work in difference form (D = 3): 3 sub, 3 fma/mul, mul, exp2, fma
//   mfma_f16   v_mfma_f32_32x32x16_f16, four independent accumulators per wavefront
//   copy       float4 copy of 4 GiB (read + write bytes per second)
// Compiled like the library: no packed FP32 instructions.
#include <hip/hip_runtime.h>

#include <cstdio>

typedef float f16v __attribute__((ext_vector_type(16)));
typedef _Float16 h8v __attribute__((ext_vector_type(8)));

#define CK(x)                                                                        \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));             \
            return 1;                                                                \
        }                                                                            \
    } while (0)

template <int MODE>
__global__ __launch_bounds__(256) void valu_rate_kernel(float *out, int iters, float s, const float *__restrict__ src) {
    float x[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) x[k] = threadIdx.x * 1e-3f + (float)k;
    for (int i = 0; i < iters; ++i) {
        if (MODE == 0) {
#pragma unroll
            for (int k = 0; k < 8; ++k) x[k] = fmaf(x[k], s, 0.5f);
        } else if (MODE == 1) {
#pragma unroll
            for (int k = 0; k < 8; ++k) x[k] = __builtin_amdgcn_exp2f(x[k]);
        } else if (MODE == 2) {   // eight chains of (exp2, fma) pairs; the values stay in [-0.5, 0.25]
#pragma unroll
            for (int k = 0; k < 8; ++k) x[k] = fmaf(__builtin_amdgcn_exp2f(x[k]), -0.5f, s - 0.749f);
        } else {                  // two pairs in difference form: lane = target, the sources wave-uniform from memory
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float *q = src + ((8 * i + 4 * h) & 255);
                const float d0 = q[0] - x[4 * h], d1 = q[1] - x[4 * h + 1], d2 = q[2] - x[4 * h + 2];
                float r = d0 * d0;
                r = fmaf(d1, d1, r);
                r = fmaf(d2, d2, r);
                x[4 * h + 3] = fmaf(__builtin_amdgcn_exp2f(r * -0.7f), q[3], x[4 * h + 3]);
            }
        }
    }
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) t += x[k];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = t;
}

__global__ __launch_bounds__(256) void mfma_rate_kernel(float *out, int iters) {
    f16v c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) c[k][v] = 0.f;
    h8v a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (_Float16)(threadIdx.x * 1e-3f);
        b[e] = (_Float16)1.0f;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int k = 0; k < 4; ++k) c[k] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c[k], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) t += c[k][v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = t;
}

__global__ __launch_bounds__(256) void copy_kernel(const float4 *__restrict__ a, float4 *__restrict__ b, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) b[i] = a[i];
}

int main() {
    hipDeviceProp_t pr;
    CK(hipGetDeviceProperties(&pr, 0));
    const int cus = pr.multiProcessorCount;
    float *out;
    CK(hipMalloc(&out, (size_t)cus * 32 * 256 * sizeof(float)));
    float *src;   // 64 sources (three coordinates and a weight each)
    CK(hipMalloc(&src, 256 * sizeof(float)));
    {
        float h[256];
        for (int k = 0; k < 256; ++k) h[k] = 0.01f * (float)((k * 37) % 101);
        CK(hipMemcpy(src, h, sizeof(h), hipMemcpyHostToDevice));
    }
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const int blocks = cus * 32, iters = 20000;   // 8 wavefronts per SIMD
    double lane_ops[4] = {0, 0, 0, 0};
    for (int mode = 0; mode < 4; ++mode) {
        float ms = 0.f;
        for (int rep = 0; rep < 3; ++rep) {
            CK(hipEventRecord(e0));
            if (mode == 0) valu_rate_kernel<0><<<blocks, 256>>>(out, iters, 0.999f, src);
            if (mode == 1) valu_rate_kernel<1><<<blocks, 256>>>(out, iters, 0.999f, src);
            if (mode == 2) valu_rate_kernel<2><<<blocks, 256>>>(out, iters, 0.999f, src);
            if (mode == 3) valu_rate_kernel<3><<<blocks, 256>>>(out, iters, 0.999f, src);
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
        }
        const double lanes = (double)blocks * 256 * iters;
        const double per_iter = mode < 3 ? 8.0 : 2.0;   // instructions, or pairs, per lane and iteration
        lane_ops[mode] = lanes * per_iter / (ms * 1e-3);
    }
    float ms = 0.f;
    for (int rep = 0; rep < 3; ++rep) {
        CK(hipEventRecord(e0));
        mfma_rate_kernel<<<cus * 8, 256>>>(out, iters);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
    }
    const double mfma_flops = (double)cus * 8 * 4 * iters * 4 * (2.0 * 32 * 32 * 16) / (ms * 1e-3);
    const size_t n = (size_t)1 << 28;   // float4: 4 GiB each way
    float4 *a, *b;
    CK(hipMalloc(&a, n * 16));
    CK(hipMalloc(&b, n * 16));
    CK(hipMemset(a, 1, n * 16));
    for (int rep = 0; rep < 3; ++rep) {
        CK(hipEventRecord(e0));
        copy_kernel<<<(unsigned)(n / 256), 256>>>(a, b, n);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
    }
    const double copy_bps = 2.0 * (double)n * 16 / (ms * 1e-3);
    const double slots = (double)cus * 64 * (double)pr.clockRate * 1e3;   // lanes x clock: one lane-slot per lane and cycle
    std::printf("{\"device\": \"%s\", \"compute_units\": %d, \"clock_mhz\": %.0f, \"lane_slots_per_s\": %.4g, "
                "\"fma_lane_ops_per_s\": %.4g, \"exp2_lane_ops_per_s\": %.4g, \"exp2_fma_pairs_per_s\": %.4g, "
                "\"difference_form_pairs_per_s\": %.4g, \"mfma_f16_32x32x16_flops\": %.4g, \"copy_bytes_per_s\": %.4g, "
                "\"cycles_per_wave_fma\": %.3g, \"cycles_per_wave_exp2\": %.3g, \"cycles_per_wave_exp2_fma_pair\": %.3g}\n",
                pr.gcnArchName, cus, pr.clockRate / 1e3, slots, lane_ops[0], lane_ops[1], lane_ops[2], lane_ops[3], mfma_flops,
                copy_bps, 4.0 * slots / lane_ops[0], 4.0 * slots / lane_ops[1], 4.0 * slots / lane_ops[2]);
    return 0;
}
