// Sustained matrix-rate probe for gfx950: a measurement aid of the benchmark, built as its own small library
// (libsawattn_probe.so) so that the attention library holds nothing but the attention path.
#include <hip/hip_runtime.h>

#include <cstdio>

#include "sawattn_probe.h"

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef unsigned u4 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*

// 16-byte chunk permutation of a 64 x 128 tile of 16-bit elements, the one the attention kernel uses for its
// K tiles (conflict-free for 16 lanes reading the same chunk of 16 consecutive rows).
__device__ __forceinline__ int swz128(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

__device__ __forceinline__ f16v mfma_f16(u4 a, u4 b, f16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
}

// What the matrix pipes of this chip sustain, to put the datasheet peak into context: every
// wavefront runs `iters` x 16 v_mfma_f32_32x32x16_f16 on four independent accumulators.
//   mode 0: all operands zero.  Nothing switches in the multipliers, the chip holds its peak clock
//           and the rate is the datasheet's.
//   mode 1: operands in registers holding values distributed like attention inputs (about
//           0.5 x standard normal); A cycles through four registers, B through four.
//   mode 2: as mode 1 with the A operands re-read from an LDS tile with the K-operand access
//           pattern of the attention kernel, one ds_read_b128 per MFMA.
// The chip is power limited and lowers its clock with switching activity, so the rate with live
// data is far below the rate with zeros, whatever the instruction stream does besides.
__device__ __forceinline__ unsigned probe_hash(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
// Two binary16 values, each about 0.5 x standard normal (sum of four uniforms, centred and scaled).
__device__ __forceinline__ unsigned probe_pair(unsigned seed) {
    h2 v;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const unsigned r = probe_hash(seed * 2u + k + 1u);
        const float u = (float)(r & 255u) + (float)((r >> 8) & 255u) + (float)((r >> 16) & 255u) + (float)(r >> 24);
        v[k] = (_Float16)((u - 510.0f) * (0.5f / 147.8f));
    }
    return __builtin_bit_cast(unsigned, v);
}

__global__ __launch_bounds__(512) void mfma_probe_kernel(float* sink, int iters, int mode) {
    __shared__ __align__(16) char tile[16384];
    LDS_PTR(char) lds = (LDS_PTR(char))tile;
    for (int i = threadIdx.x; i < 16384 / 4; i += blockDim.x) ((LDS_PTR(unsigned))lds)[i] = probe_pair(i);
    __syncthreads();
    const int lane = threadIdx.x & 63, g = lane >> 5, ln = lane & 31;
    u4 a4[4], b4[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a4[q][e] = mode == 0 ? 0u : probe_pair(100000u + threadIdx.x * 32u + q * 4u + e);
            b4[q][e] = mode == 0 ? 0u : probe_pair(900000u + threadIdx.x * 32u + q * 4u + e);
        }
    f16v c[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[q][r] = 0.f;
    unsigned addr[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) addr[ks] = (unsigned)(size_t)lds + ln * 256 + ((2 * ks + g) ^ swz128(ln)) * 16;
    if (mode != 2) {
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int t = 0; t < 16; ++t) c[t & 3] = mfma_f16(a4[t & 3], b4[(t >> 2) & 3], c[t & 3]);
        }
    } else {
        for (int i = 0; i < iters; ++i) {
            u4 a[16];
            a[0] = *(LDS_PTR(u4))(size_t)addr[0];
            a[1] = *(LDS_PTR(u4))(size_t)(addr[0] + 8192);
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                if (t + 2 < 16) a[t + 2] = *(LDS_PTR(u4))(size_t)(addr[(t + 2) / 2] + ((t + 2) & 1) * 8192);
                c[t & 3] = mfma_f16(a[t], b4[(t >> 2) & 3], c[t & 3]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    const float res = c[0][0] + c[1][1] + c[2][2] + c[3][3];
    if (res == 123.456f) sink[threadIdx.x] = res;   // never true: keeps the accumulators alive
}


thread_local char g_probe_err[160] = "";
int probe_fail(int code, const char* msg) {
    std::snprintf(g_probe_err, sizeof g_probe_err, "%s", msg);
    return code;
}

}  // namespace

extern "C" {

int sawattn_mfma_probe(float* sink, int iters, int mode, void* hip_stream, double* flops_out) {
    if (!sink || iters <= 0 || mode < 0 || mode > 2) return probe_fail(1, "sink non-null, iters > 0, mode 0, 1 or 2");
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
        (void)hipGetLastError();
        return probe_fail(3, "cannot query the device");
    }
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(cus), dim3(512), 0, static_cast<hipStream_t>(hip_stream), sink, iters, mode);
    if (hipGetLastError() != hipSuccess) return probe_fail(3, "probe launch failed");
    if (flops_out) *flops_out = (double)cus * 8.0 * (double)iters * 16.0 * (2.0 * 32 * 32 * 16);
    return 0;
}

const char* sawattn_probe_last_error(void) { return g_probe_err; }

}  // extern "C"
