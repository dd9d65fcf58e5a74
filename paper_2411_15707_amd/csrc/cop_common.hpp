// Shared host/device definitions of the COP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <type_traits>

namespace nimbus {

constexpr int kMaxLimbs = 4;
constexpr int kMaxRows = 1 << 30;     // rows of X: keeps every rounded-up row count inside an int

// Per-limb constants for the final reduction.  For a prime q with bit length b
// (2^(b-1) < q < 2^b) the reduction below takes a value V < 2^(b+63) held as
// hi:lo and returns V mod q:
//     v1   = floor(V / 2^(b-1))                     (< 2^64)
//     qhat = floor(v1 * mu / 2^64),  mu = floor(2^(b+63) / q)
// qhat never exceeds floor(V/q) and falls short of it by at most 2, so
// V - qhat*q lies in [0, 3q) and fits 64 bits because q < 2^62.
struct Limb {
    uint64_t q;
    uint64_t mu;
    uint32_t s1;        // b - 1, in [1, 61]
    uint32_t pad;
};

struct LimbTable {
    Limb limb[kMaxLimbs];
};

__device__ __forceinline__ uint64_t barrett128(uint64_t hi, uint64_t lo, const Limb &P)
{
    const uint64_t v1 = (hi << (64u - P.s1)) | (lo >> P.s1);
    const uint64_t qhat = __umul64hi(v1, P.mu);
    uint64_t r = lo - qhat * P.q;
    if (r >= P.q) r -= P.q;
    if (r >= P.q) r -= P.q;
    return r;
}

// Problem description after validation (host side).
struct Problem {
    int m, k, x_bits, n, N, L, Ch;
    size_t C;                 // Ch * 2 * L * N columns per row
    LimbTable limbs;
    int q_bits_max;           // bit length of the largest modulus
};

// ---- byte-plane (matrix core) geometry -----------------------------------
// DX signed byte planes of X, DQ signed byte planes of the centred residues.
// A value that fits fewer planes also fits more, so small parameters share the
// kernels built for DX in {2,3,4} and DQ in {7,8}.
inline int planes_x(int x_bits) { const int d = (x_bits + 7) / 8; return d < 2 ? 2 : d; }
inline int planes_q(int q_bits) { const int d = (q_bits + 1 + 7) / 8; return d < 7 ? 7 : d; }
constexpr int kTile = 32;            // rows / columns / k per matrix-core tile
constexpr int kTileBytes = 1024;     // one 32 x 32 int8 operand tile
// k is padded with zero byte planes to whole 32-value k-blocks
inline int kblocks(int k) { return (k + kTile - 1) / kTile; }

// launchers implemented in the kernel files; all return hipError_t
hipError_t launch_cop_valu(const Problem &p, const uint64_t *X, const uint64_t *ctW,
                           const uint64_t *mask, uint64_t *out, hipStream_t stream);
hipError_t launch_prepare(const Problem &p, const uint64_t *ctW, void *prepared,
                          hipStream_t stream);
hipError_t launch_stage_shares(const Problem &p, const uint64_t *X, int half_shift,
                               void *workspace, hipStream_t stream);
hipError_t launch_stage_shares_batch(const Problem &p, int count, const uint64_t *const *X,
                                     int half_shift, void *const *workspace, hipStream_t stream);
hipError_t launch_cop_mfma_batch(const Problem &p, int count, const void *const *staged,
                                 const void *const *prepared, const uint64_t *const *masks,
                                 const uint64_t *prev, uint64_t *const *outs, hipStream_t stream);
hipError_t launch_cop_mfma(const Problem &p, const void *staged, const void *prepared,
                           const uint64_t *mask, const uint64_t *prev, uint64_t *out,
                           hipStream_t stream);
bool mfma_supported(const Problem &p);
// matrix-core kernel on the canonical layout (cop_canon.hip)
bool canon_supported(const Problem &p);
hipError_t launch_cop_canon(const Problem &p, const uint64_t *X, const uint64_t *ctW,
                            const uint64_t *mask, uint64_t *out, hipStream_t stream);
hipError_t launch_cop_check(const Problem &p, const uint64_t *X, const uint64_t *ctW,
                            const uint64_t *mask, uint64_t *violations, hipStream_t stream);
hipError_t launch_cop_pack(const Problem &p, const uint64_t *rows, const uint64_t *mask,
                           uint64_t *packed, hipStream_t stream);

// Launches a kernel and returns the status of this launch alone.  (The status the runtime
// keeps per thread would also hand out, and clear, an error that an unrelated earlier call
// left behind.)
template <typename... KArgs>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream,
                         std::common_type_t<KArgs>... args)
{
    void *ptrs[] = {(void *)&args...};
    return hipLaunchKernel((const void *)kernel, grid, block, ptrs, 0, stream);
}

}  // namespace nimbus
