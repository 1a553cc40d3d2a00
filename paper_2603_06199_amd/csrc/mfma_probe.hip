// What the chip gives a bare stream of bf16 MFMAs: a measurement aid for the roofline figures,
// not part of the library.  256 CUs x 2 workgroups x 4 waves issue v_mfma_f32_32x32x16_bf16 back to
// back (four independent accumulators per wave), with the A operand either held in registers or
// read from LDS with ds_read_b128 before every MFMA, on operands with random mantissas and signs
// or on all-zero operands.  The instruction streams of the random and the zero runs are the same;
// only the operand bits differ.  Prints one JSON line.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kLdsBytes = 65536;   // per workgroup: two workgroups per CU, eight waves per CU
constexpr int kGrid = 512;

__device__ inline uint32_t mix(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// two bf16 values in (-2, -1] u [1, 2): random sign and mantissa, fixed exponent; or zeros
__device__ inline uint32_t operand_bits(uint32_t seed, bool zero) {
    return zero ? 0u : ((mix(seed) & 0x807f807fu) | 0x3f803f80u);
}

// READS: ds_read_b128 per 16 MFMAs (0 or 16); LDS_ONLY: no MFMAs, 16 reads per iteration
template <int READS, bool LDS_ONLY>
__global__ __launch_bounds__(256, 2) void probe_kernel(float *out, int iters, int zero) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, l = tid & 63, w = tid >> 6;
    for (int i = tid; i < kLdsBytes / 4; i += 256)
        reinterpret_cast<uint32_t *>(smem)[i] = operand_bits((uint32_t)i * 2654435761u + blockIdx.x, zero != 0);
    __syncthreads();
    u32x4 bw;
    for (int i = 0; i < 4; ++i) bw[i] = operand_bits((uint32_t)(tid * 4 + i) + 12345u, zero != 0);
    const bf16x8 b = __builtin_bit_cast(bf16x8, bw);
    f32x16 c[4];
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
    const char *base = smem + w * 16384 + l * 16;   // wave w reads its own 16 KB, lane-contiguous: no bank conflicts
    for (int it = 0; it < iters; ++it) {
        if (LDS_ONLY) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const u32x4 a = *reinterpret_cast<const u32x4 *>(base + j * 1024);
                asm volatile("" ::"v"(a));
            }
        } else {
            bf16x8 a = *reinterpret_cast<const bf16x8 *>(base);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (READS == 16) a = *reinterpret_cast<const bf16x8 *>(base + j * 1024);
                c[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[j & 3], 0, 0, 0);
            }
        }
        asm volatile("" ::: "memory");
    }
    float r = 0.f;
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 16; ++i) r += c[j][i];
    out[blockIdx.x * 256 + tid] = r;
}

template <int READS, bool LDS_ONLY>
double run(float *out, int iters, int zero) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.0;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(probe_kernel<READS, LDS_ONLY>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
        return -1.0;
    probe_kernel<READS, LDS_ONLY><<<kGrid, 256, kLdsBytes>>>(out, 200, zero);   // warm-up
    bool ok = hipEventRecord(e0) == hipSuccess;
    probe_kernel<READS, LDS_ONLY><<<kGrid, 256, kLdsBytes>>>(out, iters, zero);
    ok = ok && hipEventRecord(e1) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
    float ms = 0.f;
    ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (!ok) return -1.0;
    const double per_iter = (double)kGrid * 4 * iters * 16.0;     // MFMAs, or 1 KB reads
    return LDS_ONLY ? per_iter * 1024.0 / (ms * 1e9)              // TB/s
                    : per_iter * 32768.0 / (ms * 1e9);            // TFLOP/s
}

}  // namespace

int main() {
    float *out = nullptr;
    if (hipMalloc(&out, (size_t)kGrid * 256 * sizeof(float)) != hipSuccess) {
        std::fprintf(stderr, "mfma_probe: no GPU memory (is a GPU present?)\n");
        return 2;
    }
    const int iters = 40000;   // about 20 ms per run
    const double reg_rnd = run<0, false>(out, iters, 0), lds_rnd = run<16, false>(out, iters, 0);
    const double reg_zero = run<0, false>(out, iters, 1), lds_zero = run<16, false>(out, iters, 1);
    const double lds_bw = run<0, true>(out, iters, 0);
    std::printf("{\"mfma_bf16_tflops\": {\"operand_in_registers_random\": %.0f, \"operand_in_registers_zeros\": %.0f, "
                "\"operand_from_lds_random\": %.0f, \"operand_from_lds_zeros\": %.0f}, \"lds_read_b128_tb_per_s\": %.1f, "
                "\"published_peak_tflops\": 2500, \"launch\": \"512 workgroups x 4 waves, two waves per SIMD\"}\n",
                reg_rnd, reg_zero, lds_rnd, lds_zero, lds_bw);
    (void)hipFree(out);
    return reg_rnd > 0 && lds_bw > 0 ? 0 : 1;
}
