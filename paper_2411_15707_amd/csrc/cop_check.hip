// Debugging aid: counts the input words that break the value-range preconditions of the COP
// entry points (shares below 2^x_bits, residues below the modulus of their limb).
// Contract: include/nimbus_cop.h (nimbus_cop_check_inputs).
#include "cop_common.hpp"

namespace nimbus {

__global__ void check_clear_kernel(unsigned long long *violations)
{
    if (threadIdx.x < 3) violations[threadIdx.x] = 0;
}

// words of a [rows][C] residue array that are >= the modulus of their column's limb
__global__ __launch_bounds__(256) void check_residues_kernel(const uint64_t *__restrict__ a,
                                                             uint64_t total, uint32_t C, int log_n,
                                                             int L, LimbTable limbs,
                                                             unsigned long long *count)
{
    unsigned bad = 0;
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < total; i += stride) {
        const uint32_t col = (uint32_t)(i % C);
        const uint64_t q = limbs.limb[(col >> log_n) % (uint32_t)L].q;
        bad += a[i] >= q ? 1u : 0u;
    }
    // one atomic per wave
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_down(bad, off, 64);
    if ((threadIdx.x & 63) == 0 && bad) atomicAdd(count, (unsigned long long)bad);
}

__global__ __launch_bounds__(256) void check_shares_kernel(const uint64_t *__restrict__ X,
                                                           uint64_t total, int x_bits,
                                                           unsigned long long *count)
{
    unsigned bad = 0;
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < total; i += stride)
        bad += (x_bits < 64 && (X[i] >> x_bits) != 0) ? 1u : 0u;
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_down(bad, off, 64);
    if ((threadIdx.x & 63) == 0 && bad) atomicAdd(count, (unsigned long long)bad);
}

static unsigned blocks_for(uint64_t total)
{
    const uint64_t b = (total + 255u) / 256u;
    return (unsigned)(b < 1 ? 1 : (b > 4096 ? 4096 : b));
}

hipError_t launch_cop_check(const Problem &p, const uint64_t *X, const uint64_t *ctW,
                            const uint64_t *mask, uint64_t *violations, hipStream_t stream)
{
    unsigned long long *v = (unsigned long long *)violations;
    int log_n = 0;
    while ((1 << log_n) < p.N) ++log_n;
    // (a fill kernel, not a memset: callers may record this into a graph)
    hipError_t e = launch(check_clear_kernel, dim3(1), dim3(64), stream, v);
    if (e != hipSuccess) return e;
    const uint64_t nx = (uint64_t)p.m * (uint64_t)p.k;
    e = launch(check_shares_kernel, dim3(blocks_for(nx)), dim3(256), stream, X, nx, p.x_bits, v + 0);
    if (e != hipSuccess) return e;
    const uint64_t nw = (uint64_t)p.k * p.C;
    e = launch(check_residues_kernel, dim3(blocks_for(nw)), dim3(256), stream, ctW, nw,
               (uint32_t)p.C, log_n, p.L, p.limbs, v + 1);
    if (e != hipSuccess) return e;
    if (mask) {
        const uint64_t nm = (uint64_t)p.m * p.C;
        e = launch(check_residues_kernel, dim3(blocks_for(nm)), dim3(256), stream, mask, nm,
                   (uint32_t)p.C, log_n, p.L, p.limbs, v + 2);
    }
    return e;
}

}  // namespace nimbus
