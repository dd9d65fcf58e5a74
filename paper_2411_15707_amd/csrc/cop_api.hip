// C ABI of the COP library: argument validation, per-limb constants, dispatch.
// Declarations and the contract of every entry point: include/nimbus_cop.h.
#include "cop_common.hpp"
#include "../../include/nimbus_cop.h"
#include <mutex>

namespace nimbus {

// Share workspace of nimbus_cop_matmul_prepared_static: device memory that is part of the
// loaded code object, so the entry point needs no allocation.  Every GPU the library runs
// on holds its own copy at its own address until the process ends.
static __device__ __align__(256) unsigned char scratch[NIMBUS_COP_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void *scratch_ptr[kMaxDevices];          // device address of `scratch`, per device

// Device address of this device's copy of `scratch` (the array's name in host code is only a
// handle for the runtime, not an address a kernel could use).  Looked up once per device, with
// that device current.
static void *scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        scratch_ptr[dev] = ptr;
    }
    return scratch_ptr[dev];
}

static int bit_length(uint64_t v)
{
    int b = 0;
    while (v) { ++b; v >>= 1; }
    return b;
}

// Shape / modulus checks shared by every entry point.  with_x = false means "the
// call has no X" (prepare, size queries) and skips the checks that involve it.
// Shares wider than 32 bits (up to 64) are accepted here; the entry points that
// cannot handle them answer NIMBUS_COP_ERR_UNSUPPORTED.
static int make_problem(int m, int k, int x_bits, int n, int N, int L,
                        const uint64_t *moduli, bool with_x, Problem *out)
{
    if (!moduli) return NIMBUS_COP_ERR_INVALID_ARG;
    if (k < 1 || n < 1 || k >= (1 << 24)) return NIMBUS_COP_ERR_INVALID_ARG;
    if (N < 32 || N > 65536 || (N & (N - 1)) != 0) return NIMBUS_COP_ERR_INVALID_ARG;
    if (L < 1 || L > kMaxLimbs) return NIMBUS_COP_ERR_INVALID_ARG;
    if (with_x && (m < 1 || m > kMaxRows || x_bits < 1 || x_bits > 64))
        return NIMBUS_COP_ERR_INVALID_ARG;
    Problem p{};
    p.m = with_x ? m : 0;
    p.k = k;
    p.x_bits = with_x ? x_bits : 0;
    p.n = n;
    p.N = N;
    p.L = L;
    const unsigned long long Ch = ((unsigned long long)n + (unsigned)N - 1) / (unsigned)N;
    const unsigned long long C = Ch * 2ull * (unsigned)L * (unsigned)N;
    if (C >= (1ull << 31)) return NIMBUS_COP_ERR_INVALID_ARG;
    p.Ch = (int)Ch;
    p.C = (size_t)C;
    p.q_bits_max = 0;
    for (int l = 0; l < L; ++l) {
        const uint64_t q = moduli[l];
        if ((q & 1) == 0 || q >= (1ull << 62) || q < 3) return NIMBUS_COP_ERR_INVALID_ARG;
        // t < q_l for shares of up to 32 bits (wider shares exceed any single limb)
        if (with_x && x_bits <= 32 && q <= (1ull << x_bits)) return NIMBUS_COP_ERR_INVALID_ARG;
        const int b = bit_length(q);
        Limb &P = p.limbs.limb[l];
        P.q = q;
        P.s1 = (uint32_t)(b - 1);
        // mu = floor(2^(b+63) / q); b + 63 <= 125
        P.mu = (uint64_t)((((unsigned __int128)1) << (b + 63)) / q);
        P.pad = 0;
        if (b > p.q_bits_max) p.q_bits_max = b;
    }
    *out = p;
    return NIMBUS_COP_OK;
}

static size_t prepared_bytes_of(const Problem &p)
{
    const size_t CT = p.C / kTile;
    const size_t KB = (size_t)kblocks(p.k);
    const size_t DQ = (size_t)planes_q(p.q_bits_max);
    return CT * KB * DQ * kTileBytes + p.C * sizeof(uint64_t);
}

// the staging kernel indexes its threads with 32 bits
static bool staging_fits(int m, int k)
{
    const uint64_t RT = (uint64_t)(m + kTile - 1) / kTile, KB = (uint64_t)kblocks(k);
    return RT * KB <= (1ull << 23);
}

// byte ranges [a, a + na) and [b, b + nb) share a byte (a null pointer or an empty range shares none)
static bool overlaps(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b || na == 0 || nb == 0) return false;
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

// Shares of more than 32 bits are staged as two halves: the lower 32 bits first (4 byte
// planes), then the upper x_bits - 32 bits.
static size_t half_bytes(int m, int k, int half_bits)
{
    const size_t RT = (size_t)(m + kTile - 1) / kTile;
    const size_t KB = (size_t)kblocks(k);
    return RT * KB * (size_t)planes_x(half_bits) * kTileBytes;
}

static size_t workspace_bytes_of(int m, int k, int x_bits)
{
    if (x_bits <= 32) return half_bytes(m, k, x_bits);
    return half_bytes(m, k, 32) + half_bytes(m, k, x_bits - 32);
}

// the two passes of a wide share: same problem with the width of one half
static Problem half_problem(const Problem &p, int half_bits)
{
    Problem h = p;
    h.x_bits = half_bits;
    return h;
}

static bool prepared_path_supported(const Problem &p)
{
    if (p.x_bits <= 32) return mfma_supported(p);
    return mfma_supported(half_problem(p, 32)) && mfma_supported(half_problem(p, p.x_bits - 32));
}

static hipError_t stage_all(const Problem &p, const uint64_t *X, void *workspace, hipStream_t stream)
{
    if (p.x_bits <= 32) return launch_stage_shares(p, X, 0, workspace, stream);
    hipError_t e = launch_stage_shares(half_problem(p, 32), X, 0, workspace, stream);
    if (e != hipSuccess) return e;
    return launch_stage_shares(half_problem(p, p.x_bits - 32), X, 32,
                               (char *)workspace + half_bytes(p.m, p.k, 32), stream);
}

// x = x_lo + 2^32 x_hi: the pass over the upper halves writes its reduced result to out,
// the pass over the lower halves adds 2^32 times it (and the mask) and overwrites it
static hipError_t matmul_all(const Problem &p, const void *staged, const void *prepared,
                             const uint64_t *mask, uint64_t *out, hipStream_t stream)
{
    if (p.x_bits <= 32) return launch_cop_mfma(p, staged, prepared, mask, nullptr, out, stream);
    const void *staged_hi = (const char *)staged + half_bytes(p.m, p.k, 32);
    hipError_t e = launch_cop_mfma(half_problem(p, p.x_bits - 32), staged_hi, prepared, nullptr,
                                   nullptr, out, stream);
    if (e != hipSuccess) return e;
    return launch_cop_mfma(half_problem(p, 32), staged, prepared, mask, out, out, stream);
}

}  // namespace nimbus

using namespace nimbus;

extern "C" {

// checks shared by the two entry points on the canonical layout
static int canonical_problem(const uint64_t *X, int m, int k, int x_bits, const uint64_t *ctW,
                             int n, int N, int L, const uint64_t *moduli, const uint64_t *mask,
                             uint64_t *out, Problem *p)
{
    if (!X || !ctW || !out) return NIMBUS_COP_ERR_INVALID_ARG;
    const int rc = make_problem(m, k, x_bits, n, N, L, moduli, true, p);
    if (rc != NIMBUS_COP_OK) return rc;
    if (x_bits > 32) return NIMBUS_COP_ERR_UNSUPPORTED;    // wide shares: prepared path only
    if ((m + 15) / 16 > 65535) return NIMBUS_COP_ERR_UNSUPPORTED;   // grid of the vector-ALU kernel
    const size_t out_bytes = (size_t)m * p->C * sizeof(uint64_t);
    if (overlaps(out, out_bytes, X, (size_t)m * (size_t)k * sizeof(uint64_t)) ||
        overlaps(out, out_bytes, ctW, (size_t)k * p->C * sizeof(uint64_t)) ||
        overlaps(out, out_bytes, mask, out_bytes))
        return NIMBUS_COP_ERR_INVALID_ARG;
    return NIMBUS_COP_OK;
}

int nimbus_cop_matmul(const uint64_t *X, int m, int k, int x_bits,
                      const uint64_t *ctW, int n, int N, int L,
                      const uint64_t *moduli,
                      const uint64_t *mask, uint64_t *out, void *stream)
{
    Problem p;
    const int rc = canonical_problem(X, m, k, x_bits, ctW, n, N, L, moduli, mask, out, &p);
    if (rc != NIMBUS_COP_OK) return rc;
    // the matrix-core kernel where its limits allow, the vector-ALU kernel for everything else
    const hipError_t e = canon_supported(p)
                             ? launch_cop_canon(p, X, ctW, mask, out, (hipStream_t)stream)
                             : launch_cop_valu(p, X, ctW, mask, out, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

int nimbus_cop_matmul_valu(const uint64_t *X, int m, int k, int x_bits,
                           const uint64_t *ctW, int n, int N, int L,
                           const uint64_t *moduli,
                           const uint64_t *mask, uint64_t *out, void *stream)
{
    Problem p;
    const int rc = canonical_problem(X, m, k, x_bits, ctW, n, N, L, moduli, mask, out, &p);
    if (rc != NIMBUS_COP_OK) return rc;
    const hipError_t e = launch_cop_valu(p, X, ctW, mask, out, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

size_t nimbus_cop_prepared_bytes(int k, int n, int N, int L, const uint64_t *moduli)
{
    Problem p;
    if (make_problem(0, k, 0, n, N, L, moduli, false, &p) != NIMBUS_COP_OK) return 0;
    return prepared_bytes_of(p);
}

int nimbus_cop_prepare(const uint64_t *ctW, int k, int n, int N, int L,
                       const uint64_t *moduli,
                       void *prepared, size_t prepared_bytes, void *stream)
{
    if (!ctW || !prepared) return NIMBUS_COP_ERR_INVALID_ARG;
    if (((uintptr_t)prepared & 15u) != 0) return NIMBUS_COP_ERR_INVALID_ARG;
    Problem p;
    const int rc = make_problem(0, k, 0, n, N, L, moduli, false, &p);
    if (rc != NIMBUS_COP_OK) return rc;
    if (prepared_bytes < prepared_bytes_of(p)) return NIMBUS_COP_ERR_BUFFER_SIZE;
    if (overlaps(prepared, prepared_bytes_of(p), ctW, (size_t)k * p.C * sizeof(uint64_t)))
        return NIMBUS_COP_ERR_INVALID_ARG;
    const hipError_t e = launch_prepare(p, ctW, prepared, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

size_t nimbus_cop_workspace_bytes(int m, int k, int x_bits)
{
    if (m < 1 || m > kMaxRows || k < 1 || k >= (1 << 24) || x_bits < 1 || x_bits > 64) return 0;
    return workspace_bytes_of(m, k, x_bits);
}

int nimbus_cop_stage_shares(const uint64_t *X, int m, int k, int x_bits,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    if (!X || !workspace || ((uintptr_t)workspace & 15u) != 0) return NIMBUS_COP_ERR_INVALID_ARG;
    if (m < 1 || m > kMaxRows || k < 1 || k >= (1 << 24) || x_bits < 1 || x_bits > 64)
        return NIMBUS_COP_ERR_INVALID_ARG;
    if (!staging_fits(m, k)) return NIMBUS_COP_ERR_UNSUPPORTED;
    if (workspace_bytes < workspace_bytes_of(m, k, x_bits)) return NIMBUS_COP_ERR_BUFFER_SIZE;
    if (overlaps(workspace, workspace_bytes_of(m, k, x_bits), X, (size_t)m * (size_t)k * sizeof(uint64_t)))
        return NIMBUS_COP_ERR_INVALID_ARG;
    Problem p{};
    p.m = m;
    p.k = k;
    p.x_bits = x_bits;
    const hipError_t e = stage_all(p, X, workspace, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

int nimbus_cop_stage_shares_batch(int count, const uint64_t *const *X, int m, int k, int x_bits,
                                  void *const *workspaces, size_t workspace_bytes, void *stream)
{
    if (count < 1 || count > NIMBUS_COP_MAX_BATCH || !X || !workspaces)
        return NIMBUS_COP_ERR_INVALID_ARG;
    if (m < 1 || m > kMaxRows || k < 1 || k >= (1 << 24) || x_bits < 1 || x_bits > 64)
        return NIMBUS_COP_ERR_INVALID_ARG;
    if (x_bits > 32) return NIMBUS_COP_ERR_UNSUPPORTED;      // wide shares: two halves per problem
    if (!staging_fits(m, k)) return NIMBUS_COP_ERR_UNSUPPORTED;
    const size_t need = workspace_bytes_of(m, k, x_bits), x_bytes = (size_t)m * (size_t)k * sizeof(uint64_t);
    if (workspace_bytes < need) return NIMBUS_COP_ERR_BUFFER_SIZE;
    for (int i = 0; i < count; ++i)
        if (!X[i] || !workspaces[i] || ((uintptr_t)workspaces[i] & 15u) != 0)
            return NIMBUS_COP_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i)
        for (int j = 0; j < count; ++j)
            if (overlaps(workspaces[i], need, X[j], x_bytes) ||
                (i != j && overlaps(workspaces[i], need, workspaces[j], need)))
                return NIMBUS_COP_ERR_INVALID_ARG;
    Problem p{};
    p.m = m;
    p.k = k;
    p.x_bits = x_bits;
    const hipError_t e = launch_stage_shares_batch(p, count, X, 0, workspaces, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

int nimbus_cop_matmul_staged(const void *staged_shares, int m, int k, int x_bits,
                             const void *prepared, int n, int N, int L,
                             const uint64_t *moduli,
                             const uint64_t *mask, uint64_t *out, void *stream)
{
    if (!staged_shares || !prepared || !out) return NIMBUS_COP_ERR_INVALID_ARG;
    if ((((uintptr_t)prepared | (uintptr_t)staged_shares) & 15u) != 0)
        return NIMBUS_COP_ERR_INVALID_ARG;
    Problem p;
    const int rc = make_problem(m, k, x_bits, n, N, L, moduli, true, &p);
    if (rc != NIMBUS_COP_OK) return rc;
    if (!prepared_path_supported(p)) return NIMBUS_COP_ERR_UNSUPPORTED;
    const size_t out_bytes = (size_t)m * p.C * sizeof(uint64_t);
    if (overlaps(out, out_bytes, staged_shares, workspace_bytes_of(m, k, x_bits)) ||
        overlaps(out, out_bytes, prepared, prepared_bytes_of(p)) ||
        overlaps(out, out_bytes, mask, out_bytes))
        return NIMBUS_COP_ERR_INVALID_ARG;
    const hipError_t e = matmul_all(p, staged_shares, prepared, mask, out, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

int nimbus_cop_matmul_staged_batch(int count, const void *const *staged_shares, int m, int k,
                                   int x_bits, const void *const *prepared, int n, int N, int L,
                                   const uint64_t *moduli, const uint64_t *const *masks,
                                   uint64_t *const *outs, void *stream)
{
    if (count < 1 || count > NIMBUS_COP_MAX_BATCH || !staged_shares || !prepared || !outs)
        return NIMBUS_COP_ERR_INVALID_ARG;
    if (x_bits > 32) return NIMBUS_COP_ERR_UNSUPPORTED;      // wide shares: two passes per problem
    Problem p;
    const int rc = make_problem(m, k, x_bits, n, N, L, moduli, true, &p);
    if (rc != NIMBUS_COP_OK) return rc;
    if (!prepared_path_supported(p)) return NIMBUS_COP_ERR_UNSUPPORTED;
    // tile ids of the whole launch are 32-bit
    const uint64_t tiles = (uint64_t)(p.C / 64) * (uint64_t)((m + 127) / 128) * (uint64_t)count;
    if (tiles >= (1ull << 31)) return NIMBUS_COP_ERR_UNSUPPORTED;
    const size_t out_bytes = (size_t)m * p.C * sizeof(uint64_t);
    const size_t ws_bytes = workspace_bytes_of(m, k, x_bits), prep_bytes = prepared_bytes_of(p);
    const uint64_t *no_masks[NIMBUS_COP_MAX_BATCH] = {};
    for (int i = 0; i < count; ++i) {
        if (!staged_shares[i] || !prepared[i] || !outs[i]) return NIMBUS_COP_ERR_INVALID_ARG;
        if ((((uintptr_t)prepared[i] | (uintptr_t)staged_shares[i]) & 15u) != 0)
            return NIMBUS_COP_ERR_INVALID_ARG;
        if (masks && (masks[i] == nullptr) != (masks[0] == nullptr))
            return NIMBUS_COP_ERR_INVALID_ARG;                // a mask for every problem or for none
    }
    // no output may overlap anything another problem (or its own) reads or writes
    for (int i = 0; i < count; ++i)
        for (int j = 0; j < count; ++j) {
            if (overlaps(outs[i], out_bytes, staged_shares[j], ws_bytes) ||
                overlaps(outs[i], out_bytes, prepared[j], prep_bytes) ||
                (masks && overlaps(outs[i], out_bytes, masks[j], out_bytes)) ||
                (i != j && overlaps(outs[i], out_bytes, outs[j], out_bytes)))
                return NIMBUS_COP_ERR_INVALID_ARG;
        }
    const hipError_t e = launch_cop_mfma_batch(p, count, staged_shares, prepared,
                                               masks ? masks : no_masks, nullptr, outs,
                                               (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

// shared by the two entry points that stage and multiply in one call
static int matmul_prepared_impl(const uint64_t *X, int m, int k, int x_bits,
                                const void *prepared, int n, int N, int L,
                                const uint64_t *moduli,
                                const uint64_t *mask, uint64_t *out,
                                void *workspace, size_t workspace_bytes, bool use_static,
                                void *stream)
{
    // use_static: the workspace is the library's own buffer; its address is looked up only
    // after every check that needs no device has passed
    if (!X || !prepared || !out || (!use_static && !workspace)) return NIMBUS_COP_ERR_INVALID_ARG;
    if ((((uintptr_t)prepared | (uintptr_t)workspace) & 15u) != 0)
        return NIMBUS_COP_ERR_INVALID_ARG;
    Problem p;
    const int rc = make_problem(m, k, x_bits, n, N, L, moduli, true, &p);
    if (rc != NIMBUS_COP_OK) return rc;
    if (!prepared_path_supported(p) || !staging_fits(m, k)) return NIMBUS_COP_ERR_UNSUPPORTED;
    if (workspace_bytes < workspace_bytes_of(m, k, x_bits))
        return use_static ? NIMBUS_COP_ERR_STATIC_LIMIT : NIMBUS_COP_ERR_BUFFER_SIZE;
    if (use_static) {
        workspace = scratch_of_current_device();
        if (!workspace) return NIMBUS_COP_ERR_LAUNCH;
    }
    {
        // both written buffers against everything that is read, and against each other
        const size_t out_bytes = (size_t)m * p.C * sizeof(uint64_t);
        const size_t ws_bytes = workspace_bytes_of(m, k, x_bits);
        const size_t x_bytes = (size_t)m * (size_t)k * sizeof(uint64_t);
        if (overlaps(out, out_bytes, X, x_bytes) || overlaps(out, out_bytes, mask, out_bytes) ||
            overlaps(out, out_bytes, prepared, prepared_bytes_of(p)) ||
            overlaps(out, out_bytes, workspace, ws_bytes) ||
            overlaps(workspace, ws_bytes, X, x_bytes) || overlaps(workspace, ws_bytes, mask, out_bytes) ||
            overlaps(workspace, ws_bytes, prepared, prepared_bytes_of(p)))
            return NIMBUS_COP_ERR_INVALID_ARG;
    }
    hipError_t e = stage_all(p, X, workspace, (hipStream_t)stream);
    if (e != hipSuccess) return NIMBUS_COP_ERR_LAUNCH;
    e = matmul_all(p, workspace, prepared, mask, out, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

int nimbus_cop_matmul_prepared(const uint64_t *X, int m, int k, int x_bits,
                               const void *prepared, int n, int N, int L,
                               const uint64_t *moduli,
                               const uint64_t *mask, uint64_t *out,
                               void *workspace, size_t workspace_bytes,
                               void *stream)
{
    return matmul_prepared_impl(X, m, k, x_bits, prepared, n, N, L, moduli, mask, out, workspace,
                                workspace_bytes, false, stream);
}

int nimbus_cop_matmul_prepared_static(const uint64_t *X, int m, int k, int x_bits,
                                      const void *prepared, int n, int N, int L,
                                      const uint64_t *moduli,
                                      const uint64_t *mask, uint64_t *out,
                                      void *stream)
{
    return matmul_prepared_impl(X, m, k, x_bits, prepared, n, N, L, moduli, mask, out, nullptr,
                                (size_t)NIMBUS_COP_STATIC_WORKSPACE_BYTES, true, stream);
}

int nimbus_cop_packed_count(int m, int n, int N)
{
    if (m < 1 || m > kMaxRows || n < 1 || N < 32 || N > 65536 || (N & (N - 1)) != 0 || n > N)
        return 0;
    const int P = N / n;
    return (m + P - 1) / P;
}

int nimbus_cop_pack(const uint64_t *rows, int m, int n, int N, int L,
                    const uint64_t *moduli,
                    const uint64_t *mask, uint64_t *packed, void *stream)
{
    if (!rows || !packed || rows == packed) return NIMBUS_COP_ERR_INVALID_ARG;
    if (m < 1 || m > kMaxRows) return NIMBUS_COP_ERR_INVALID_ARG;
    Problem p;
    const int rc = make_problem(0, 1, 0, n, N, L, moduli, false, &p);
    if (rc != NIMBUS_COP_OK) return rc;
    if (n > N) return NIMBUS_COP_ERR_UNSUPPORTED;          // several ring chunks: nothing to pack
    if (nimbus_cop_packed_count(m, n, N) > 65535) return NIMBUS_COP_ERR_UNSUPPORTED;   // grid limit
    {
        const size_t ct_bytes = 2u * (size_t)L * (size_t)N * sizeof(uint64_t);    // one ciphertext
        const size_t packed_bytes = (size_t)nimbus_cop_packed_count(m, n, N) * ct_bytes;
        if (overlaps(packed, packed_bytes, rows, (size_t)m * ct_bytes) ||
            overlaps(packed, packed_bytes, mask, packed_bytes))
            return NIMBUS_COP_ERR_INVALID_ARG;
    }
    p.m = m;
    const hipError_t e = launch_cop_pack(p, rows, mask, packed, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

int nimbus_cop_check_inputs(const uint64_t *X, int m, int k, int x_bits,
                            const uint64_t *ctW, int n, int N, int L,
                            const uint64_t *moduli,
                            const uint64_t *mask, uint64_t *violations, void *stream)
{
    if (!X || !ctW || !violations) return NIMBUS_COP_ERR_INVALID_ARG;
    Problem p;
    const int rc = make_problem(m, k, x_bits, n, N, L, moduli, true, &p);
    if (rc != NIMBUS_COP_OK) return rc;
    const hipError_t e = launch_cop_check(p, X, ctW, mask, violations, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

const char *nimbus_cop_strerror(int status)
{
    switch (status) {
    case NIMBUS_COP_OK: return "ok";
    case NIMBUS_COP_ERR_INVALID_ARG: return "invalid argument (null pointer, size or modulus out of range)";
    case NIMBUS_COP_ERR_UNSUPPORTED: return "parameters not supported by this entry point";
    case NIMBUS_COP_ERR_LAUNCH: return "HIP kernel launch failed";
    case NIMBUS_COP_ERR_BUFFER_SIZE: return "prepared or workspace buffer too small";
    case NIMBUS_COP_ERR_STATIC_LIMIT:
        return "shares need more than the built-in workspace of nimbus_cop_matmul_prepared_static";
    default: return "unknown status";
    }
}

int nimbus_cop_version(void) { return 121; }

}  // extern "C"
