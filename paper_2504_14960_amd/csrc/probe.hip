// Measurement probe, not part of the layer: how fast this GPU issues the bf16
// matrix instruction of the grouped GEMM when nothing else is in the way.
//
// Every workgroup copies a 64 KiB operand image into LDS once (256 rows of 64
// bf16 values for each of the two operands, rows of 128 bytes, 16-byte pieces
// XOR-swizzled by the row as in the GEMM kernels) and then loops over it: four
// waves, each with a 128 x 128 accumulator block, read their fragments from LDS
// and issue 32x32x16 MFMAs, with no global memory traffic, no barrier and no
// epilogue in the loop.  The rate depends on the VALUES in the image: all-zero
// operands run at the published peak, operands distributed like the workload's
// (activations ~N(0,1), weights ~N(0,0.02^2)) draw more power and the clock
// falls; the kernel reports the shader clock it ran at next to the elapsed time
// the caller measures.
#include "common.h"

namespace moe {

namespace {

__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(const uint32_t* __restrict__ image, int iters,
                                                              float* __restrict__ sink,
                                                              unsigned long long* __restrict__ ticks) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 65536 / 16; i += 256)
        reinterpret_cast<u32x4*>(lds)[i] = reinterpret_cast<const u32x4*>(image)[i];
    __syncthreads();
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int fr = lane & 31, fk = lane >> 5;
    const int row_a = (wave >> 1) * 128 + fr, row_b = (wave & 1) * 128 + fr;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int piece = 2 * ks + fk;
            bf16x8 a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = row_a + 32 * i;
                a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(lds + r * 128 + ((piece ^ lds_swizzle(r)) << 4)));
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = row_b + 32 * j;
                b[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(lds + 32768 + r * 128 + ((piece ^ lds_swizzle(r)) << 4)));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
    if (ticks && blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = __builtin_amdgcn_s_memtime() - c0;       // shader clocks
        ticks[1] = __builtin_amdgcn_s_memrealtime() - r0;   // 100 MHz reference clocks
    }
}

typedef __attribute__((ext_vector_type(8))) int probe_i32x8;

// The same loop for the FP8 path: rows of 128 E4M3 bytes, every lane feeds 32
// consecutive bytes of a row (two 16-byte pieces) to a 32x32x64 MFMA, two
// k-steps per pass over the image.
__global__ __launch_bounds__(256) void probe_mfma_fp8_kernel(const uint32_t* __restrict__ image, int iters,
                                                             float* __restrict__ sink,
                                                             unsigned long long* __restrict__ ticks) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 65536 / 16; i += 256)
        reinterpret_cast<u32x4*>(lds)[i] = reinterpret_cast<const u32x4*>(image)[i];
    __syncthreads();
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int fr = lane & 31, fk = lane >> 5;
    const int row_a = (wave >> 1) * 128 + fr, row_b = (wave & 1) * 128 + fr;
    auto frag = [&](const uint8_t* base, int r, int ks) -> probe_i32x8 {
        const int piece = 4 * ks + 2 * fk;
        const u32x4 lo = *reinterpret_cast<const u32x4*>(base + r * 128 + ((piece ^ lds_swizzle(r)) << 4));
        const u32x4 hi = *reinterpret_cast<const u32x4*>(base + r * 128 + (((piece + 1) ^ lds_swizzle(r)) << 4));
        probe_i32x8 v;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            v[t] = (int)lo[t];
            v[4 + t] = (int)hi[t];
        }
        return v;
    };
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            probe_i32x8 a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = frag(lds, row_a + 32 * i, ks);
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = frag(lds + 32768, row_b + 32 * j, ks);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[j], a[i], acc[i][j], 0, 0, 0, 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
    if (ticks && blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = __builtin_amdgcn_s_memtime() - c0;
        ticks[1] = __builtin_amdgcn_s_memrealtime() - r0;
    }
}

}  // namespace

void launch_probe_mfma_fp8(const void* image, int iters, int workgroups, float* sink, unsigned long long* ticks,
                           hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(probe_mfma_fp8_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
        attr_set = true;
    }
    hipLaunchKernelGGL(probe_mfma_fp8_kernel, dim3(workgroups), dim3(256), 65536, s,
                       static_cast<const uint32_t*>(image), iters, sink, ticks);
}

void launch_probe_mfma_bf16(const void* image, int iters, int workgroups, float* sink, unsigned long long* ticks,
                            hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(probe_mfma_bf16_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
        attr_set = true;
    }
    hipLaunchKernelGGL(probe_mfma_bf16_kernel, dim3(workgroups), dim3(256), 65536, s,
                       static_cast<const uint32_t*>(image), iters, sink, ticks);
}

}  // namespace moe
