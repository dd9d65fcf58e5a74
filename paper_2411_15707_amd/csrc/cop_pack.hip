// Output packing by right shifts (Algorithm 1 step 3; Appendix B.1 "Right Shift"), with the
// mask of step 4 applied to the packed ciphertexts.
//
// RShift(ct, s) multiplies both polynomials of a ciphertext by X^s in Z_q[X]/(X^N+1):
// coefficient c moves to c+s, a coefficient that passes the end re-enters at c+s-N negated.
// With P = floor(N/n) rows per packed ciphertext,
//   packed[theta] = sum_{u<P} RShift(rows[theta P + u], u n) + mask[theta]   (mod q_l),
// rows past m counting as zero.  Seen from the output: coefficient c of packed[theta] is
//   sum_u  sign * rows[theta P + u][(c - u n) mod N],   sign = -1 where c < u n,
// a gather of P words, so one thread owns one output coefficient of one polynomial and limb
// and no two threads write the same word.  Bound by HBM: every input word is read once
// (consecutive threads read consecutive words), every output word written once.
#include "cop_common.hpp"

namespace nimbus {

struct PackArgs {
    const uint64_t *rows;     // [m][2][L][N]
    const uint64_t *mask;     // [T][2][L][N] or nullptr
    uint64_t *packed;         // [T][2][L][N]
    int m, n, N, L, P, T;
    uint64_t q[kMaxLimbs];
};

// W consecutive words per thread (1, or 2 as one 16-byte access where every shift u n is even
// and the buffers are 16-byte aligned: both words of a pair then move together and wrap
// together).  CH rows are loaded at a time (2 where a packed ciphertext holds at most two).
template <int W, int CH>
__global__ __launch_bounds__(256) void cop_pack_kernel(const PackArgs a)
{
    typedef uint64_t Words __attribute__((ext_vector_type(W)));
    // grid: x covers the 2 L N words of one packed ciphertext, y = theta
    const uint32_t w = (blockIdx.x * 256u + threadIdx.x) * (uint32_t)W;       // first word inside the ciphertext
    const uint32_t words = 2u * (uint32_t)a.L * (uint32_t)a.N;
    if (w >= words) return;
    const int theta = (int)blockIdx.y;
    const uint32_t c = w & (uint32_t)(a.N - 1);               // N is a power of two
    const uint32_t block = w - c;                              // (poly, limb) offset
    const uint64_t q = a.q[(w / (uint32_t)a.N) % (uint32_t)a.L];
    auto words_at = [](const uint64_t *p) { return *(const Words *)p; };

    // every load of a thread is on its way before the first one is used: the mask's now, the
    // rows' CH at a time (a row past the last one reads the last one again and counts as zero)
    Words mk = 0;
    if (a.mask) mk = words_at(a.mask + (size_t)theta * words + w);
    uint64_t acc[W];
#pragma unroll
    for (int i = 0; i < W; ++i) acc[i] = 0;
    const int first = theta * a.P;
    const int count = a.m - first < a.P ? a.m - first : a.P;   // rows of this packed ciphertext, >= 1
    for (int u0 = 0; u0 < count; u0 += CH) {
        Words v[CH];
        bool wrapped[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int u = u0 + j < count ? u0 + j : count - 1;
            const uint32_t shift = (uint32_t)u * (uint32_t)a.n;   // < N
            wrapped[j] = c < shift;
            const uint32_t src = wrapped[j] ? c + (uint32_t)a.N - shift : c - shift;
            v[j] = words_at(a.rows + (size_t)(first + u) * words + block + src);
        }
#pragma unroll
        for (int j = 0; j < CH; ++j) {
#pragma unroll
            for (int i = 0; i < W; ++i) {
                uint64_t t = u0 + j < count ? v[j][i] : 0;
                if (wrapped[j] && t != 0) t = q - t;
                acc[i] += t;                                   // both below q < 2^62
                if (acc[i] >= q) acc[i] -= q;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < W; ++i) {
        uint64_t t = mk[i];
        if (t >= q) t -= q;                                    // tolerate an unreduced mask word
        acc[i] += t;
        if (acc[i] >= q) acc[i] -= q;
    }
    Words r;
#pragma unroll
    for (int i = 0; i < W; ++i) r[i] = acc[i];
    *(Words *)(a.packed + (size_t)theta * words + w) = r;
}

hipError_t launch_cop_pack(const Problem &p, const uint64_t *rows, const uint64_t *mask,
                           uint64_t *packed, hipStream_t stream)
{
    PackArgs a{};
    a.rows = rows;
    a.mask = mask;
    a.packed = packed;
    a.m = p.m;
    a.n = p.n;
    a.N = p.N;
    a.L = p.L;
    a.P = p.N / p.n;
    a.T = (p.m + a.P - 1) / a.P;
    for (int l = 0; l < p.L; ++l) a.q[l] = p.limbs.limb[l].q;
    const uint32_t words = 2u * (uint32_t)p.L * (uint32_t)p.N;
    const bool pairs = p.n % 2 == 0 &&
                       (((uintptr_t)rows | (uintptr_t)mask | (uintptr_t)packed) & 15u) == 0;
    const dim3 grid((words / (pairs ? 2 : 1) + 255) / 256, (uint32_t)a.T), block(256);
    if (a.P <= 2)
        return pairs ? launch(cop_pack_kernel<2, 2>, grid, block, stream, a)
                     : launch(cop_pack_kernel<1, 2>, grid, block, stream, a);
    return pairs ? launch(cop_pack_kernel<2, 4>, grid, block, stream, a)
                 : launch(cop_pack_kernel<1, 4>, grid, block, stream, a);
}

}  // namespace nimbus
