// Peak probes for the benchmark (not part of liblqer): what this chip delivers for the two resources the
// forward pass is priced against (Sec. 2.1: the memory-bound and the compute-bound regime), measured with
// kernels that do nothing else.
//   lqer_probe_stream_read  reads a buffer once with the access pattern of the weight stream: every wavefront
//                           issues contiguous 1 KiB loads (16 bytes per lane, streaming hint), several in flight
//   lqer_probe_copy         plain copy, 16 bytes per lane (read + write traffic)
//   lqer_probe_mfma         register-resident loop of 32x32x16 bf16 MFMAs, `chains` independent accumulators
//                           per wavefront, `waves` wavefronts per SIMD on every compute unit
//   lqer_probe_mfma_random  the same with operands of random signs and significands
//   lqer_probe_mfma_valu    the same loop (bf16 32x32x16 or int8 32x32x32) with a fixed number of independent fp32
//                           vector instructions behind every MFMA: what the matrix pipe still delivers when a kernel
//                           has that much vector work per MFMA (both kinds of instruction issue through one port)
// All launches are asynchronous on the given stream; the caller times them with events.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// UNROLL = 1 KiB loads a wavefront keeps in flight
template <int UNROLL>
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, int64_t n_kib, uint32_t* sink) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    u32x4 acc = u32x4{0, 0, 0, 0};
    // wavefront w takes the 1 KiB pieces w, w + nwaves, ... : at any moment the chip reads one contiguous range
    int64_t i = wave;
    for (; i + (UNROLL - 1) * nwaves < n_kib; i += UNROLL * nwaves) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) v[j] = __builtin_nontemporal_load(src + (i + j * nwaves) * 64 + lane);
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) acc ^= v[j];
    }
    for (; i < n_kib; i += nwaves) acc ^= __builtin_nontemporal_load(src + i * 64 + lane);
    // never true for the buffers the benchmark passes (all ones would be needed): keeps the loads alive
    if ((acc[0] & acc[1] & acc[2] & acc[3]) == 0xFFFFFFFFu && sink != nullptr) sink[0] = acc[0];
}

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// RANDOM: operands with random signs and significands (values in +-[1, 2)), four different pairs used in turn, instead
// of one pair of small non-negative integers: the same instruction stream with the data toggling as it does in a real
// product, which is what the chip's power management reacts to.
template <int CHAINS, bool RANDOM>
__global__ __launch_bounds__(256) void mfma_kernel(int iters, float* sink) {
    f32x16 acc[CHAINS];
#pragma unroll
    for (int c = 0; c < CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    union Op { bf16x8 v; uint16_t h[8]; };
    Op a[4], b[4];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (RANDOM) {
                uint32_t x = (threadIdx.x * 8u + e) * 2654435761u + p * 40503u + blockIdx.x * 2246822519u;
                x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
                a[p].h[e] = (uint16_t)(0x3F80u | (x & 0x807Fu));
                b[p].h[e] = (uint16_t)(0x3F80u | ((x >> 16) & 0x807Fu));
            } else {
                a[p].v[e] = (__bf16)(float)((threadIdx.x + e) & 3);
                b[p].v[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
            }
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < CHAINS; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c & 3].v, b[(c + (c >> 2)) & 3].v, acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) s += acc[c][0] + acc[c][15];
    if (s == -1.2345f && sink != nullptr) sink[0] = s;       // keeps the arithmetic alive; not a value these sums take
}

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

// Four independent accumulators; NV fused multiply-adds on registers of their own behind every MFMA.  The
// instructions are written as asm statements so that they stay in this order.
template <int NV, bool I8>
__global__ __launch_bounds__(256) void mfma_valu_kernel(int iters, float* sink, float y, float z) {
    constexpr int CH = 4;
    f32x16 acc[CH];
    i32x16 iacc[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc[c][r] = 0.f;
            iacc[c][r] = 0;
        }
    bf16x8 a, b;
    i32x4 ia, ib;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)((threadIdx.x + e) & 3);
        b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        ia[e] = (int)threadIdx.x + e;
        ib[e] = (int)threadIdx.x * 3 + e;
    }
    float v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = (float)(threadIdx.x + j);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            if constexpr (I8) asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+v"(iacc[c]) : "v"(ia), "v"(ib));
            else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[c]) : "v"(a), "v"(b));
#pragma unroll
            for (int j = 0; j < NV; ++j) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(v[(c * NV + j) & 15]) : "v"(y), "v"(z));
        }
    }
    asm volatile("s_nop 15\n s_nop 15");           // the last MFMAs' results are read below: past their latency
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) s += acc[c][0] + acc[c][15] + (float)iacc[c][3];
#pragma unroll
    for (int j = 0; j < 16; ++j) s += v[j];
    if (s == -1.2345f && sink != nullptr) sink[0] = s;    // keeps the arithmetic alive; not a value these sums take
}

template <bool I8>
int launch_mfma_valu(int workgroups, int iters, int valu, float* sink, hipStream_t s) {
    const dim3 grid((unsigned)workgroups), block(256);
    switch (valu) {
        case 0: hipLaunchKernelGGL((mfma_valu_kernel<0, I8>), grid, block, 0, s, iters, sink, 1.0f, 0.0f); break;
        case 4: hipLaunchKernelGGL((mfma_valu_kernel<4, I8>), grid, block, 0, s, iters, sink, 1.0f, 0.0f); break;
        case 8: hipLaunchKernelGGL((mfma_valu_kernel<8, I8>), grid, block, 0, s, iters, sink, 1.0f, 0.0f); break;
        case 12: hipLaunchKernelGGL((mfma_valu_kernel<12, I8>), grid, block, 0, s, iters, sink, 1.0f, 0.0f); break;
        default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

}  // namespace

extern "C" {

// bytes: multiple of 1024; in_flight: 4, 8 or 16 loads of 1 KiB per wavefront.  Returns 0, or the hipError_t of the launch.
int lqer_probe_stream_read(const void* src_dev, int64_t bytes, void* sink_dev, int workgroups, int in_flight, void* hip_stream) {
    if (!src_dev || bytes <= 0 || (bytes & 1023) != 0 || workgroups <= 0) return (int)hipErrorInvalidValue;
    const dim3 grid((unsigned)workgroups), block(256);
    hipStream_t s = (hipStream_t)hip_stream;
    const u32x4* src = (const u32x4*)src_dev;
    uint32_t* sink = (uint32_t*)sink_dev;
    if (in_flight == 4) hipLaunchKernelGGL(stream_read_kernel<4>, grid, block, 0, s, src, bytes >> 10, sink);
    else if (in_flight == 8) hipLaunchKernelGGL(stream_read_kernel<8>, grid, block, 0, s, src, bytes >> 10, sink);
    else if (in_flight == 16) hipLaunchKernelGGL(stream_read_kernel<16>, grid, block, 0, s, src, bytes >> 10, sink);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

// bytes: multiple of 16.
int lqer_probe_copy(const void* src_dev, void* dst_dev, int64_t bytes, int workgroups, void* hip_stream) {
    if (!src_dev || !dst_dev || bytes <= 0 || (bytes & 15) != 0 || workgroups <= 0) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream,
                       (const u32x4*)src_dev, (u32x4*)dst_dev, bytes >> 4);
    return (int)hipGetLastError();
}

// Launches workgroups x 4 wavefronts, each doing iters x chains MFMAs (32 x 32 x 16, 32768 flops each).
// chains: 4 or 8.  flops of the launch = workgroups * 4 * iters * chains * 32768.
int lqer_probe_mfma(int workgroups, int iters, int chains, void* sink_dev, void* hip_stream) {
    if (workgroups <= 0 || iters <= 0) return (int)hipErrorInvalidValue;
    if (chains == 4) hipLaunchKernelGGL((mfma_kernel<4, false>), dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, (float*)sink_dev);
    else if (chains == 8) hipLaunchKernelGGL((mfma_kernel<8, false>), dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, (float*)sink_dev);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

// The same with operands whose bits differ from MFMA to MFMA and from lane to lane (see mfma_kernel).
int lqer_probe_mfma_random(int workgroups, int iters, int chains, void* sink_dev, void* hip_stream) {
    if (workgroups <= 0 || iters <= 0) return (int)hipErrorInvalidValue;
    if (chains == 4) hipLaunchKernelGGL((mfma_kernel<4, true>), dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, (float*)sink_dev);
    else if (chains == 8) hipLaunchKernelGGL((mfma_kernel<8, true>), dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, (float*)sink_dev);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

// Launches workgroups x 4 wavefronts, each doing iters x 4 MFMAs with `valu` (0, 4, 8 or 12) fp32 vector instructions
// behind each one.  int8 = 0: bf16 32x32x16 (32768 flops per MFMA); 1: int8 32x32x32 (65536 operations).
int lqer_probe_mfma_valu(int workgroups, int iters, int valu, int int8, void* sink_dev, void* hip_stream) {
    if (workgroups <= 0 || iters <= 0) return (int)hipErrorInvalidValue;
    return int8 ? launch_mfma_valu<true>(workgroups, iters, valu, (float*)sink_dev, (hipStream_t)hip_stream)
                : launch_mfma_valu<false>(workgroups, iters, valu, (float*)sink_dev, (hipStream_t)hip_stream);
}

}  // extern "C"
