// Register-only probe of what bounds a stream of v_mfma_f32_32x32x16_bf16 mixed with fp32 VALU
// instructions on one gfx950 SIMD: no memory, no LDS, operands fixed.  It is the yardstick the
// measured kernels of this library are read against (the score sweep issues 4 VALU instructions per
// matrix instruction, the attention consumer about 5).  A stand-alone executable; it is not part of
// the library and the library does not depend on it.
//
// A "slot" is one pass of the inner body: at most one matrix instruction and NV fma instructions.
// Every workgroup has 4 x W waves (W per SIMD), one workgroup per compute unit.

#include <hip/hip_runtime.h>

#include <cstdio>
#include <type_traits>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

enum Mix {
    kChain,        // matrix instructions only, each depending on the one before (one accumulator)
    kIndependent,  // matrix instructions only, four accumulators in turn
    kValuOnly,     // NV fma per slot, no matrix instruction
    kInterleaved,  // one matrix instruction (four accumulators in turn) and NV fma per slot, one wave's stream
    kSplitRoles,   // the first wave of each SIMD issues only matrix instructions, the second only NV fma per slot
    kSweepAndValu  // the first wave of each SIMD issues one matrix instruction + 4 fma per slot, the second NV fma per slot
};

template <bool MFMA, int NV, bool CHAIN>
__device__ __forceinline__ void stream(floatx16 (&acc)[4], float (&v)[8], bf16x8 a, bf16x8 b, int iters) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if constexpr (MFMA) {
                const int c = CHAIN ? 0 : (u & 3);
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
            }
#pragma unroll
            for (int n = 0; n < NV; ++n) v[n & 7] = __builtin_fmaf(v[n & 7], 1.0001f, 0.25f);
        }
    }
}

template <int MIX, int NV>
__global__ __launch_bounds__(512) void probe_kernel(float* out, int iters) {
    const int lane = threadIdx.x & 63;
    const bool first = ((threadIdx.x >> 8) & 1) == 0;  // waves 0-3: the first wave of SIMD 0-3
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = static_cast<__bf16>(0.001f * (lane + i));
        b[i] = static_cast<__bf16>(0.002f * (lane - i));
    }
    floatx16 acc[4];
    for (int c = 0; c < 4; ++c)
        for (int j = 0; j < 16; ++j) acc[c][j] = 0.0f;
    float v[8];
    for (int i = 0; i < 8; ++i) v[i] = 0.5f + lane * 0.001f + i;

    if constexpr (MIX == kChain) stream<true, 0, true>(acc, v, a, b, iters);
    else if constexpr (MIX == kIndependent) stream<true, 0, false>(acc, v, a, b, iters);
    else if constexpr (MIX == kValuOnly) stream<false, NV, false>(acc, v, a, b, iters);
    else if constexpr (MIX == kInterleaved) stream<true, NV, false>(acc, v, a, b, iters);
    else if constexpr (MIX == kSplitRoles) {
        if (first) stream<true, 0, false>(acc, v, a, b, iters);
        else stream<false, NV, false>(acc, v, a, b, iters);
    } else {
        if (first) stream<true, 4, false>(acc, v, a, b, iters);
        else stream<false, NV, false>(acc, v, a, b, iters);
    }

    float s = 0.0f;  // keeps every result alive
    for (int c = 0; c < 4; ++c)
        for (int j = 0; j < 16; ++j) s += acc[c][j];
    for (int i = 0; i < 8; ++i) s += v[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int MIX, int NV>
bool run(const char* what, int waves_per_simd, float* out, int compute_units) {
    constexpr int kIters = 20000;
    const int threads = 64 * 4 * waves_per_simd;
    hipEvent_t t0, t1;
    if (hipEventCreate(&t0) != hipSuccess || hipEventCreate(&t1) != hipSuccess) return false;
    hipLaunchKernelGGL((probe_kernel<MIX, NV>), dim3(compute_units), dim3(threads), 0, 0, out, 16);  // warm-up
    if (hipDeviceSynchronize() != hipSuccess) return false;
    if (hipEventRecord(t0) != hipSuccess) return false;
    hipLaunchKernelGGL((probe_kernel<MIX, NV>), dim3(compute_units), dim3(threads), 0, 0, out, kIters);
    if (hipEventRecord(t1) != hipSuccess || hipEventSynchronize(t1) != hipSuccess) return false;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, t0, t1) != hipSuccess) return false;
    const double ns_per_slot = ms * 1e6 / (kIters * 8.0);
    std::printf("%-62s waves/SIMD %d  fma/slot %d : %7.3f ms  %6.1f ns per slot and wave  %6.1f ns per slot and SIMD\n",
                what, waves_per_simd, NV, ms, ns_per_slot, ns_per_slot / waves_per_simd);
    std::fflush(stdout);
    return hipEventDestroy(t0) == hipSuccess && hipEventDestroy(t1) == hipSuccess;
}

}  // namespace

int main() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
        std::fprintf(stderr, "issue_probe: no GPU\n");
        return 2;
    }
    float* out = nullptr;
    if (hipMalloc(&out, static_cast<size_t>(cus) * 512 * sizeof(float)) != hipSuccess) return 2;
    std::printf("issue_probe: %d compute units, one workgroup each; 160,000 slots per wave\n", cus);
    bool ok = true;
    for (int w = 1; w <= 2 && ok; ++w) {
        ok = ok && run<kChain, 0>("matrix instructions, one dependent chain", w, out, cus);
        ok = ok && run<kIndependent, 0>("matrix instructions, four accumulators", w, out, cus);
        ok = ok && run<kValuOnly, 4>("fma only", w, out, cus);
        ok = ok && run<kValuOnly, 7>("fma only", w, out, cus);
        ok = ok && run<kInterleaved, 4>("one matrix instruction + fma per slot, same wave", w, out, cus);
        ok = ok && run<kInterleaved, 5>("one matrix instruction + fma per slot, same wave", w, out, cus);
        ok = ok && run<kInterleaved, 7>("one matrix instruction + fma per slot, same wave", w, out, cus);
        ok = ok && run<kInterleaved, 11>("one matrix instruction + fma per slot, same wave", w, out, cus);
    }
    ok = ok && run<kSplitRoles, 4>("wave A matrix instructions only, wave B fma only", 2, out, cus);
    ok = ok && run<kSplitRoles, 7>("wave A matrix instructions only, wave B fma only", 2, out, cus);
    ok = ok && run<kSweepAndValu, 7>("wave A matrix instruction + 4 fma, wave B fma only", 2, out, cus);
    ok = ok && run<kSweepAndValu, 11>("wave A matrix instruction + 4 fma, wave B fma only", 2, out, cus);
    ok = hipFree(out) == hipSuccess && ok;
    return ok ? 0 : 1;
}
