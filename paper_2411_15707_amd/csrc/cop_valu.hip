// Vector-ALU kernel for the COP accumulation on the canonical ciphertext layout
// (Algorithm 1 step 2 and step 4 of the paper): one thread owns one coefficient
// column and RT token rows, walks the k weight ciphertexts once, and keeps the
// sum unreduced until the end.
//
// Exactness of the lazy accumulation.  A residue c = c_hi * 2^32 + c_lo and a
// share x < 2^x_bits give x*c = x*c_lo + 2^32 * x*c_hi.  Within a block of
// kblk = 2^(32 - x_bits) terms
//     sum x*c_lo < kblk * 2^x_bits * 2^32 = 2^64     and
//     sum x*c_hi < kblk * 2^x_bits * 2^30 = 2^62     (c < 2^62),
// so both 64-bit partial sums are exact; after each block they are folded into
// a 128-bit total, which is reduced once (Barrett) after the mask is added.
#include "cop_common.hpp"

namespace nimbus {

__device__ __forceinline__ void add128(uint64_t &hi, uint64_t &lo, uint64_t ahi, uint64_t alo)
{
    const uint64_t s = lo + alo;
    hi += ahi + (s < lo ? 1u : 0u);
    lo = s;
}

template <int RT>
__global__ __launch_bounds__(256) void cop_valu_kernel(
    const uint64_t *__restrict__ X, int m, int k, int kblk,
    const uint64_t *__restrict__ ctW, uint32_t C, int N, int L, LimbTable limbs,
    const uint64_t *__restrict__ mask, uint64_t *__restrict__ out)
{
    const uint32_t col = blockIdx.x * 256u + threadIdx.x;
    if (col >= C) return;
    const int j0 = blockIdx.y * RT;
    const Limb P = limbs.limb[(col / (uint32_t)N) % (uint32_t)L];

    uint64_t t_lo[RT], t_hi[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) { t_lo[r] = 0; t_hi[r] = 0; }

    // rows past m read row m-1 (their sums are discarded at the store)
    const uint64_t *xrow[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const int j = (j0 + r < m) ? (j0 + r) : (m - 1);
        xrow[r] = X + (size_t)j * k;
    }

    for (int i0 = 0; i0 < k; i0 += kblk) {
        const int i1 = (i0 + kblk < k) ? (i0 + kblk) : k;
        uint64_t s_lo[RT], s_hi[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) { s_lo[r] = 0; s_hi[r] = 0; }
#pragma unroll 4
        for (int i = i0; i < i1; ++i) {
            const uint64_t c = ctW[(size_t)i * C + col];
            const uint32_t c_lo = (uint32_t)c, c_hi = (uint32_t)(c >> 32);
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const uint32_t x = (uint32_t)xrow[r][i];      // uniform over the block
                s_lo[r] += (uint64_t)x * c_lo;
                s_hi[r] += (uint64_t)x * c_hi;
            }
        }
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            add128(t_hi[r], t_lo[r], 0, s_lo[r]);
            add128(t_hi[r], t_lo[r], s_hi[r] >> 32, s_hi[r] << 32);
        }
    }

#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const int j = j0 + r;
        if (j < m) {
            const size_t idx = (size_t)j * C + col;
            uint64_t hi = t_hi[r], lo = t_lo[r];
            if (mask) add128(hi, lo, 0, mask[idx]);
            out[idx] = barrett128(hi, lo, P);
        }
    }
}

hipError_t launch_cop_valu(const Problem &p, const uint64_t *X, const uint64_t *ctW,
                           const uint64_t *mask, uint64_t *out, hipStream_t stream)
{
    constexpr int RT = 16;
    const int sh = 32 - p.x_bits;                   // x_bits in [1, 32]
    const int kblk = 1 << (sh > 30 ? 30 : sh);
    dim3 grid((unsigned)((p.C + 255) / 256), (unsigned)((p.m + RT - 1) / RT));
    return launch(cop_valu_kernel<RT>, grid, dim3(256), stream,
                  X, p.m, p.k, kblk, ctW, (uint32_t)p.C, p.N, p.L, p.limbs, mask, out);
}

}  // namespace nimbus
