// Calibration kernels for the benchmark: what this chip sustains on the two resources the
// COP kernel leans on, measured the same way the kernel uses them.  Not part of the COP
// path; declared in include/nimbus_calib.h.
//
//  * int8 matrix-core rate: a register-only loop of v_mfma_i32_32x32x32_i8 with three A
//    operands, seven B operands and nine accumulators per wave (the COP kernel's 3 x 7
//    digit products), with zero or with random operand bytes.  The sustained rate depends
//    on the operand values (the chip lowers its clock under load), so both are measured.
//  * HBM read rate: a grid-stride read of a buffer with 16-byte loads.
//  * butterfly rate: a register-only loop of the number-theoretic transform's butterfly as
//    the server-side kernels compute it (Appendix B.1: ciphertext polynomials are multiplied
//    in the transform domain), eight values and three stages per thread: what the vector
//    ALUs sustain on that mix of 64-bit integer work when no memory is involved.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "cop_common.hpp"
#include "../../include/nimbus_calib.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ inline uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

__global__ __launch_bounds__(256) void calib_mfma_kernel(int iters, int random_operands, int *sink)
{
    v4i a[3], b[7];
    const uint32_t seed = blockIdx.x * 256u + threadIdx.x;
    for (int i = 0; i < 3; ++i)
        for (int r = 0; r < 4; ++r)
            a[i][r] = random_operands ? (int)mix32(seed * 31u + (uint32_t)(i * 4 + r) + 1u) : 0;
    for (int i = 0; i < 7; ++i)
        for (int r = 0; r < 4; ++r)
            b[i][r] = random_operands ? (int)mix32(seed * 77u + (uint32_t)(i * 4 + r) + 1000u) : 0;
    v16i c[9];
    for (int i = 0; i < 9; ++i)
        for (int r = 0; r < 16; ++r) c[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 21; ++i)
            c[i / 7 + i % 7] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i / 7], b[i % 7],
                                                                    c[i / 7 + i % 7], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < 9; ++i) s += c[i][0];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void calib_read_kernel(const u32x4 *__restrict__ src, size_t n16,
                                                         uint32_t *sink)
{
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * 256u;
    for (size_t i = (size_t)blockIdx.x * 256u + threadIdx.x; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;      // keeps the loads alive, (almost) never taken
}

// The butterflies of the transform kernels, the same arithmetic written out here so that the
// calibration stands on its own; w a table value, ws = floor(w 2^64 / q).
//   LOOSE = false: Harvey-style lazy butterfly on values < 4q for any q < 2^62, one conditional
//                  subtraction;
//   LOOSE = true:  what the kernels do for 2^34 <= q < 2^58: no conditional subtraction, and the
//                  quotient of the product estimated from three of the four partial products
//                  (nq = 2^64 - q: the difference becomes a sum that the multiply-add chain
//                  absorbs).  Values are left to wrap in this loop: it measures a rate, its
//                  results mean nothing.
template <bool LOOSE>
__device__ __forceinline__ void butterfly(uint64_t &a, uint64_t &b, uint64_t w, uint64_t ws,
                                          uint64_t q, uint64_t two_q, uint64_t nq)
{
    if constexpr (LOOSE) {
        const uint32_t b0 = (uint32_t)b, b1 = (uint32_t)(b >> 32);
        const uint32_t w0 = (uint32_t)ws, w1 = (uint32_t)(ws >> 32);
        const uint64_t h = (uint64_t)b1 * w1 + __umulhi(b0, w1) + __umulhi(b1, w0);
        const uint64_t u = a, v = b * w + h * nq;
        a = u + v;
        b = u + 2 * two_q - v;
    } else {
        const uint64_t u = a >= two_q ? a - two_q : a;
        const uint64_t v = b * w - __umul64hi(b, ws) * q;
        a = u + v;
        b = u - v + two_q;
    }
}

template <bool LOOSE>
__global__ __launch_bounds__(256) void calib_butterfly_kernel(int iters, uint64_t q, uint64_t *sink)
{
    const uint32_t seed = blockIdx.x * 256u + threadIdx.x;
    uint64_t x[8], w[7], ws[7];
    for (int i = 0; i < 8; ++i) x[i] = (((uint64_t)mix32(seed * 8u + i) << 32) | mix32(seed + 77u * i)) % q;
    for (int i = 0; i < 7; ++i) {
        w[i] = (((uint64_t)mix32(seed * 7u + i + 100u) << 32) | mix32(seed + 13u * i)) % q;
        ws[i] = (uint64_t)(((unsigned __int128)w[i] << 64) / q);
    }
    const uint64_t two_q = 2 * q;
    uint64_t nq = 0 - q;
    asm volatile("" : "+s"(nq));        // keeps the sum a sum
    for (int it = 0; it < iters; ++it) {
        // stages of distance 4, 2, 1 over the thread's eight values: 12 butterflies
#pragma unroll
        for (int st = 0; st < 3; ++st) {
            const int half = 4 >> st;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                if (r & half) continue;
                const int t = (1 << st) - 1 + (r >> (3 - st));
                butterfly<LOOSE>(x[r], x[r + half], w[t], ws[t], q, two_q, nq);
            }
        }
    }
    uint64_t s = 0;
    for (int i = 0; i < 8; ++i) s ^= x[i];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" {

long long nimbus_calib_mfma_i8(int workgroups, int iters, int random_operands, void *sink,
                               size_t sink_bytes, void *stream)
{
    if (workgroups < 1 || workgroups > 65535 || iters < 1 || !sink) return -1;
    if (sink_bytes < (size_t)workgroups * 256u * sizeof(int)) return -1;
    if (nimbus::launch(calib_mfma_kernel, dim3((uint32_t)workgroups), dim3(256), (hipStream_t)stream,
                       iters, random_operands, (int *)sink) != hipSuccess)
        return -1;
    // int8 operations issued: 4 waves x iters x 21 instructions x 2 * 32*32*32 each
    return (long long)workgroups * 4ll * iters * 21ll * 65536ll;
}

long long nimbus_calib_stream_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink || bytes < 16 || ((uintptr_t)src & 15u) != 0) return -1;
    const size_t n16 = bytes / 16;
    if (nimbus::launch(calib_read_kernel, dim3(256 * 16), dim3(256), (hipStream_t)stream,
                       (const u32x4 *)src, n16, (uint32_t *)sink) != hipSuccess)
        return -1;
    return (long long)(n16 * 16);
}

long long nimbus_calib_butterflies(int workgroups, int iters, unsigned long long q, void *sink,
                                   size_t sink_bytes, void *stream)
{
    if (workgroups < 1 || workgroups > 65535 || iters < 1 || !sink) return -1;
    if (q < 3 || (q & 1u) == 0 || q >= (1ull << 62)) return -1;
    if (sink_bytes < (size_t)workgroups * 256u * sizeof(uint64_t)) return -1;
    // the butterfly that the transform kernels run for this modulus
    const bool loose = q >= (1ull << 34) && q < (1ull << 58);
    void (*const kernel)(int, uint64_t, uint64_t *) =
        loose ? calib_butterfly_kernel<true> : calib_butterfly_kernel<false>;
    if (nimbus::launch(kernel, dim3((uint32_t)workgroups), dim3(256), (hipStream_t)stream, iters,
                       (uint64_t)q, (uint64_t *)sink) != hipSuccess)
        return -1;
    return (long long)workgroups * 256ll * iters * 12ll;
}

}  // extern "C"
