// Measurement aids for the benchmark, built into their own small library (librf_probe.so) so that the
// product library exports nothing but the paper's operations.  What the chip sustains on
// v_mfma_f32_32x32x16_bf16 alone, and on the attention kernel's instruction mix without any memory
// traffic or dependences, are the yardsticks the attention kernel's MFMA fraction is read against.
#include <hip/hip_runtime.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kMfmaPerIter = 32;

// MIX = 0: 32 independent-enough MFMAs per iteration (4 accumulation chains).
// MIX = 1: after every MFMA the per-MFMA VALU work of the attention kernel's softmax: one exp2 and
//          four ordinary fp32 operations on values that do not depend on the MFMAs.
template <int MIX>
__global__ void __launch_bounds__(512) probe_kernel(float* out, int iters) {
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i) acc[i] = f32x16{0};
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = static_cast<__bf16>(threadIdx.x * 0.001f);
        b[i] = static_cast<__bf16>(0.5f);
    }
    float x[10];
    for (int i = 0; i < 10; ++i) x[i] = -1.0f - 0.01f * static_cast<float>(threadIdx.x + i);
    const float c1 = 0.999f, c2 = -0.001f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kMfmaPerIter; ++i) {
            acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i & 3], 0, 0, 0);
            if (MIX) {  // five independent registers per MFMA, alternating between two sets
                float* v = x + 5 * (i & 1);
                asm volatile("v_fma_f32 %0, %0, %5, %6\n\tv_exp_f32 %1, %1\n\tv_add_f32 %2, %2, %6\n\tv_max_f32 %3, %3, %6\n\t"
                             "v_fma_f32 %4, %4, %5, %6"
                             : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4])
                             : "v"(c1), "v"(c2));
            }
        }
    }
    float r = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 16; ++j) r += acc[i][j];
    for (int i = 0; i < 10; ++i) r += x[i];
    out[blockIdx.x * 512 + threadIdx.x] = r;
}

}  // namespace

extern "C" {

// Launches the probe on `stream`: one workgroup of 8 wavefronts per CU (`cus` of them), each wavefront
// issuing iters * 32 MFMAs.  out: device, float [cus * 512].  Returns a hipError_t (0 = ok).
int rf_probe_launch(int mix, int cus, int iters, float* out, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (cus < 1 || iters < 1 || !out) return static_cast<int>(hipErrorInvalidValue);
    if (mix) hipLaunchKernelGGL(probe_kernel<1>, dim3(cus), dim3(512), 0, st, out, iters);
    else hipLaunchKernelGGL(probe_kernel<0>, dim3(cus), dim3(512), 0, st, out, iters);
    return static_cast<int>(hipGetLastError());
}

// Floating-point operations of one launch: 2 * 32 * 32 * 16 per MFMA per wavefront.
double rf_probe_flops(int cus, int iters) { return 2.0 * 32 * 32 * 16 * kMfmaPerIter * static_cast<double>(iters) * 8.0 * cus; }

}  // extern "C"
