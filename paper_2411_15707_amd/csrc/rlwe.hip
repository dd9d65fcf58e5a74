// Server side of the Nimbus linear layer on gfx950: negacyclic number-theoretic transform
// per RNS limb, and on top of it the setup-phase encryption of the weight rows (Algorithm 1
// step 1 with the row-wise encoding of Section 3.2, Eq. (2)) and the decryption + decoding
// of returned ciphertexts (Algorithm 1 step 5; Enc / Dec of Appendix B.1).
// Declarations and the contract of every entry point: include/nimbus_rlwe.h.
//
// One workgroup transforms one polynomial of one limb entirely inside the LDS:
//   load -> forward rounds -> pointwise product with the transformed secret -> inverse
//   rounds -> (add c0 | assemble c0) -> store,
// so a product c1 * s costs one read of c1 and one write of the result in HBM.  (A ring of
// 2^15 coefficients does not fit: two workgroups per polynomial take one half each, with
// the first forward stage done on the way in and the last inverse stage in a pass of its
// own; see Part below.)
//
// Transform (the usual in-place pair for X^N + 1, psi a primitive 2N-th root of unity):
//   forward:  stages m = 1, 2, 4, ..., N/2 blocks; in block i of a stage every pair
//             (j, j + t), t = N / 2m, becomes (u + w v, u - w v) with w = psi^brv(m + i);
//             natural order in, bit-reversed order out;
//   inverse:  the same stages backwards, (u, v) -> (u + v, (u - v) w^-1); the factor 1/N
//             is folded into the table of the transformed secret.
// A round keeps 2^S coefficients of a thread in registers for S <= 4 consecutive stages;
// between rounds the coefficients go through the LDS.  The last forward round, the
// pointwise product and the first inverse round work on the same coefficients of the same
// thread and are one round.  The first round takes its coefficients straight from the
// coalesced loads and the last one hands its own to the stores (one group per thread: the
// same coefficients), and rounds that keep every wave inside its own coefficients follow
// each other without a workgroup barrier.
//
// Arithmetic: a product by a table constant w uses its companion w' = floor(w 2^64 / q):
//   x w - floor(x w' / 2^64) q  lies in [0, 2q) for every 64-bit x.
// Moduli below 2^62: values kept lazily in [0, 4q) (forward) and [0, 2q) (inverse) by one
// conditional subtraction per butterfly.  Moduli from 2^34 to 2^58 (every parameter set of
// the benchmark configurations): no conditional subtractions, bounds tracked at compile time
// instead, and a cheaper quotient estimate; see group_butterflies.
//
// Tables: the constants of a transform are read once per polynomial from the second-level
// cache; they are stored a second and third time in the order in which the threads of the
// product kernels read them (neighbouring lanes, neighbouring entries; see power_slot()).
#include "rlwe_kernels.hpp"

namespace nimbus {

__device__ uint64_t powmod(uint64_t base, uint32_t e, const Limb &P)
{
    uint64_t r = 1;
    while (e) {
        if (e & 1u) r = mulmod(r, base, P);
        base = mulmod(base, base, P);
        e >>= 1;
    }
    return r;
}

// floor(w * 2^64 / q) for w < q < 2^62: schoolbook binary division
__device__ uint64_t companion(uint64_t w, uint64_t q)
{
    uint64_t r = w, quo = 0;
    for (int i = 0; i < 64; ++i) {
        r <<= 1;
        quo <<= 1;
        if (r >= q) {
            r -= q;
            quo |= 1u;
        }
    }
    return quo;
}

// ---------------------------------------------------------------------------
// setup: powers of psi in bit-reversed order, forward and inverse, with companions
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rlwe_powers_kernel(RlweArgs a, int logN, int L,
                                                          Twiddle *__restrict__ tables)
{
    const uint32_t N = 1u << logN;
    const uint32_t gid = blockIdx.x * 256u + threadIdx.x;
    if (gid >= N * (uint32_t)L) return;
    const uint32_t l = gid >> logN, i = gid & (N - 1u);
    const RlweLimb &P = a.limb[l];
    const uint32_t e = __brev(i) >> (32 - logN);
    Twiddle *const t = tables + (size_t)l * limb_table_entries((int)N);
    const uint64_t f = powmod(P.psi, e, P.red), g = powmod(P.psi_inv, e, P.red);
    t[i] = Twiddle{f, companion(f, P.red.q)};
    t[N + i] = Twiddle{g, companion(g, P.red.q)};
}

// ---------------------------------------------------------------------------
// setup: transform of the secret, times 1/N, with companions
// one workgroup per limb
// ---------------------------------------------------------------------------
template <int LOGN, int PRE>
__global__ __launch_bounds__(threads_for(LOGN - PRE, 4)) void rlwe_secret_kernel(
    RlweArgs a, const int8_t *__restrict__ s, Twiddle *__restrict__ tables)
{
    constexpr int N = 1 << LOGN, NP = N >> PRE, NT = threads_for(LOGN - PRE, 4);
    __shared__ uint64_t lds[padded_size(NP)];
    const int tid = threadIdx.x, l = blockIdx.x >> PRE, h = blockIdx.x & ((1 << PRE) - 1);
    const RlweLimb &P = a.limb[l];
    const uint64_t q = P.red.q;
    const Mod md = make_mod(P);
    Twiddle *const t = tables + (size_t)l * limb_table_entries(N);
    auto lifted = [&](int c) -> uint64_t {
        const int v = s[c];
        return v < 0 ? q - (uint64_t)(-v) : (uint64_t)v;
    };
    if constexpr (PRE == 0) {
        for (int c = tid; c < N; c += NT) lds[pad(c)] = lifted(c);
    } else {
        const Twiddle w0 = t[1];                            // stage 0 has one block: entry 1
        for (int c = tid; c < NP; c += NT)
            lds[pad(c)] = enter_part<PRE>(lifted(c), lifted(c + NP), w0, md, h);
    }
    __syncthreads();
    forward_only<LOGN, PRE, 4, PRE, NT>(lds, t, md, tid, h);
    for (int c = tid; c < NP; c += NT) {
        uint64_t v = lds[pad(c)];               // [0, 4q)
        v = v >= 2 * q ? v - 2 * q : v;
        v = v >= q ? v - q : v;
        v = mulmod(v, P.n_inv, P.red);
        t[2 * N + h * NP + c] = Twiddle{v, companion(v, q)};
    }
}

// setup: set 0 of every limb copied into the order of the product kernels with `maxs` stages
// per round (see power_slot()); one thread per entry
__global__ __launch_bounds__(256) void rlwe_table_set_kernel(Twiddle *__restrict__ tables, int logN, int L,
                                                             int pre, int maxs, int set)
{
    const uint32_t N = 1u << logN;
    const uint32_t gid = blockIdx.x * 256u + threadIdx.x;
    if (gid >= N * (uint32_t)L) return;
    const uint32_t l = gid >> logN, e = gid & (N - 1u);
    const Twiddle *const from = tables + (size_t)l * limb_table_entries((int)N);
    Twiddle *const to = tables + (size_t)l * limb_table_entries((int)N) + (size_t)set * set_entries((int)N);
    const int p = power_slot(logN, pre, maxs, (int)e);
    to[p] = from[e];
    to[N + p] = from[N + e];
    to[2 * N + secret_slot(logN, pre, maxs, (int)e)] = from[2 * N + e];
}

// ---------------------------------------------------------------------------
// decoding: CRT of the limb phases, then rounding division by Delta
// ---------------------------------------------------------------------------
struct DecodeArgs {
    const uint64_t *phi;    // [T][L][N]
    uint64_t *m_hat;        // [T][N]
    int L, logN;
    uint64_t total;         // T * N
    uint64_t q0;
    Limb red1;              // limb 1 (L == 2)
    uint64_t q0_inv;        // q0^-1 mod q1
    uint64_t delta_hi, delta_lo, half_hi, half_lo;   // Delta and floor(Delta / 2)
    double delta_inv;       // 1 / Delta, rounded
    uint64_t t_mask;
};

__global__ __launch_bounds__(256) void rlwe_decode_kernel(DecodeArgs a)
{
    const uint64_t gid = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (gid >= a.total) return;
    const uint64_t N = 1ull << a.logN;
    const uint64_t row = gid >> a.logN, c = gid & (N - 1);
    const uint64_t *const ph = a.phi + row * (uint64_t)a.L * N;
    const uint64_t p0 = ph[c];
    u128 v = p0;
    if (a.L == 2) {
        // Garner: phi = p0 + q0 * ((p1 - p0) * q0^-1 mod q1)
        const uint64_t q1 = a.red1.q;
        const uint64_t p1 = ph[N + c];
        const uint64_t p0r = barrett128(0, p0, a.red1);
        uint64_t diff = p1 + q1 - p0r;
        diff = diff >= q1 ? diff - q1 : diff;
        const uint64_t h = mulmod(diff, a.q0_inv, a.red1);
        v += (u128)a.q0 * h;
    }
    const u128 delta = ((u128)a.delta_hi << 64) | a.delta_lo;
    const u128 num = v + (((u128)a.half_hi << 64) | a.half_lo);
    // quotient <= 2^32 + 1: a double-precision estimate is within one of it
    const double nd = fma((double)(uint64_t)(num >> 64), 18446744073709551616.0,
                          (double)(uint64_t)num);
    uint64_t est = (uint64_t)(nd * a.delta_inv);
    u128 prod = delta * est;                    // about num: no overflow
    if (prod > num) {                           // one too many
        est -= 1;
        prod -= delta;
    }
    if (num - prod >= delta) est += 1;          // one too few
    a.m_hat[gid] = est & a.t_mask;
}

// The same for three and four limbs: Q < 2^248, so the reconstructed phase and Delta take
// four 64-bit words (least significant first).  Mixed-radix form of the Chinese remainder
// theorem: phi = a_0 + q_0 (a_1 + q_1 (a_2 + q_2 a_3)) with
//   a_j = ( ... ((phi_j - a_0) q_0^-1 - a_1) q_1^-1 - ... - a_{j-1}) q_{j-1}^-1  mod q_j,
// all of it 64-bit modular arithmetic; only the final Horner evaluation is wide.
struct Wide {
    uint64_t w[4];
};

__device__ __forceinline__ Wide wide_mul_add(const Wide &a, uint64_t m, uint64_t add)   // a m + add
{
    Wide r;
    u128 carry = add;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const u128 p = (u128)a.w[i] * m + carry;
        r.w[i] = (uint64_t)p;
        carry = p >> 64;
    }
    return r;
}

__device__ __forceinline__ Wide wide_add(const Wide &a, const Wide &b)
{
    Wide r;
    u128 carry = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const u128 t = (u128)a.w[i] + b.w[i] + carry;
        r.w[i] = (uint64_t)t;
        carry = t >> 64;
    }
    return r;
}

// a - b modulo 2^256 and whether it borrowed (a < b)
__device__ __forceinline__ bool wide_sub(const Wide &a, const Wide &b, Wide &r)
{
    uint64_t borrow = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const u128 t = (u128)a.w[i] - b.w[i] - borrow;
        r.w[i] = (uint64_t)t;
        borrow = (uint64_t)(t >> 64) & 1u;
    }
    return borrow != 0;
}

struct DecodeWideArgs {
    const uint64_t *phi;    // [T][L][N]
    uint64_t *m_hat;        // [T][N]
    int L, logN;            // L = 3 or 4
    uint64_t total;         // T * N
    Limb red[kMaxLimbs];
    uint64_t inv[kMaxLimbs][kMaxLimbs];     // inv[i][j] = q_i^-1 mod q_j for i < j
    Wide delta, half;       // Delta and floor(Delta / 2)
    double delta_inv;       // 1 / Delta, rounded
    uint64_t t_mask;
};

__global__ __launch_bounds__(256) void rlwe_decode_wide_kernel(DecodeWideArgs a)
{
    const uint64_t gid = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (gid >= a.total) return;
    const uint64_t N = 1ull << a.logN;
    const uint64_t row = gid >> a.logN, c = gid & (N - 1);
    const uint64_t *const ph = a.phi + row * (uint64_t)a.L * N + c;
    uint64_t digit[kMaxLimbs] = {0, 0, 0, 0};
    digit[0] = ph[0];
#pragma unroll
    for (int j = 1; j < kMaxLimbs; ++j) {
        if (j >= a.L) break;
        const Limb &P = a.red[j];
        uint64_t v = ph[(uint64_t)j * N];
#pragma unroll
        for (int i = 0; i < j; ++i) {
            const uint64_t d = barrett128(0, digit[i], P);      // a_i mod q_j
            v = v + P.q - d;
            v = v >= P.q ? v - P.q : v;
            v = mulmod(v, a.inv[i][j], P);
        }
        digit[j] = v;
    }
    Wide v = {{a.L == 4 ? digit[3] : 0, 0, 0, 0}};
    if (a.L == 4) v = wide_mul_add(v, a.red[2].q, digit[2]);
    else v.w[0] = digit[2];
    v = wide_mul_add(v, a.red[1].q, digit[1]);
    v = wide_mul_add(v, a.red[0].q, digit[0]);
    const Wide num = wide_add(v, a.half);
    // quotient <= 2^32 + 1: a double-precision estimate is within one of it
    const double two64 = 18446744073709551616.0;
    double nd = (double)num.w[3];
    nd = fma(nd, two64, (double)num.w[2]);
    nd = fma(nd, two64, (double)num.w[1]);
    nd = fma(nd, two64, (double)num.w[0]);
    uint64_t est = (uint64_t)(nd * a.delta_inv);
    Wide prod = wide_mul_add(a.delta, est, 0);  // about num: no overflow
    Wide rem;
    if (wide_sub(num, prod, rem)) {             // one too many
        est -= 1;
        rem = wide_add(rem, a.delta);           // wraps back to num - (est) Delta
    }
    Wide over;
    if (!wide_sub(rem, a.delta, over)) est += 1;    // one too few
    a.m_hat[gid] = est & a.t_mask;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static uint64_t h_mulmod(uint64_t a, uint64_t b, uint64_t q) { return (uint64_t)((u128)a * b % q); }

static uint64_t h_powmod(uint64_t base, uint64_t e, uint64_t q)
{
    uint64_t r = 1 % q;
    base %= q;
    while (e) {
        if (e & 1) r = h_mulmod(r, base, q);
        base = h_mulmod(base, base, q);
        e >>= 1;
    }
    return r;
}

// inverse of a modulo mod (coprime), by the extended Euclidean algorithm
static uint64_t h_invmod(uint64_t a, uint64_t mod)
{
    __int128 old_r = (__int128)(a % mod), r = (__int128)mod, old_c = 1, c = 0;
    while (r != 0) {
        const __int128 quo = old_r / r;
        const __int128 nr = old_r - quo * r;
        old_r = r;
        r = nr;
        const __int128 ncoef = old_c - quo * c;
        old_c = c;
        c = ncoef;
    }
    if (old_r != 1) return 0;                   // not coprime
    __int128 res = old_c % (__int128)mod;
    if (res < 0) res += mod;
    return (uint64_t)res;
}

static int log2_exact(int N)
{
    int b = 0;
    while ((1 << b) < N) ++b;
    return b;
}

static int bit_length64(uint64_t v)
{
    int b = 0;
    while (v) { ++b; v >>= 1; }
    return b;
}

// shape and modulus checks shared by every entry point; fills the reduction constants
// byte ranges [a, a + na) and [b, b + nb) share a byte
static bool ranges_overlap(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b || na == 0 || nb == 0) return false;
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

static int rlwe_check(int N, int L, const uint64_t *moduli, RlweArgs *out)
{
    if (!moduli) return NIMBUS_COP_ERR_INVALID_ARG;
    if (N < 32 || N > 65536 || (N & (N - 1)) != 0) return NIMBUS_COP_ERR_INVALID_ARG;
    if (L < 1 || L > kMaxLimbs) return NIMBUS_COP_ERR_INVALID_ARG;
    RlweArgs a{};
    for (int l = 0; l < L; ++l) {
        const uint64_t q = moduli[l];
        if ((q & 1) == 0 || q >= (1ull << 62) || q < 3) return NIMBUS_COP_ERR_INVALID_ARG;
        if ((q - 1) % (2ull * (uint64_t)N) != 0) return NIMBUS_COP_ERR_INVALID_ARG;
        for (int j = 0; j < l; ++j)
            if (moduli[j] == q) return NIMBUS_COP_ERR_INVALID_ARG;
        const int b = bit_length64(q);
        Limb &P = a.limb[l].red;
        P.q = q;
        P.s1 = (uint32_t)(b - 1);
        P.mu = (uint64_t)((((u128)1) << (b + 63)) / q);
        P.pad = 0;
        if (b >= 35) {                  // fold(): only the kernels for moduli from 2^34 use it
            a.limb[l].fold_k = (uint32_t)(b - 33);
            a.limb[l].fold_m = (uint32_t)((((u128)1) << (64 + (b - 33))) / q);
        }
    }
    if (N > (1 << kRlweMaxLogN)) return NIMBUS_COP_ERR_UNSUPPORTED;
    *out = a;
    return NIMBUS_COP_OK;
}

// a primitive 2N-th root of unity: psi^N = -1.  Any of them gives the same products.
static bool find_psi(uint64_t q, int N, uint64_t *psi)
{
    const uint64_t e = (q - 1) / (2ull * (uint64_t)N);
    for (uint64_t g = 2; g < 2000 && g < q; ++g) {
        const uint64_t cand = h_powmod(g, e, q);
        if (h_powmod(cand, (uint64_t)N, q) == q - 1) {
            *psi = cand;
            return true;
        }
    }
    return false;
}

// Q and Delta = floor(Q / 2^t_bits) as four 64-bit words, least significant first
struct HostWide {
    uint64_t w[4] = {0, 0, 0, 0};
};

static HostWide hw_times(const HostWide &a, uint64_t m)
{
    HostWide r;
    u128 carry = 0;
    for (int i = 0; i < 4; ++i) {
        const u128 p = (u128)a.w[i] * m + carry;
        r.w[i] = (uint64_t)p;
        carry = p >> 64;
    }
    return r;
}

static HostWide hw_shift_right(const HostWide &a, int s)       // 0 < s < 64
{
    HostWide r;
    for (int i = 0; i < 4; ++i) {
        r.w[i] = a.w[i] >> s;
        if (i + 1 < 4) r.w[i] |= a.w[i + 1] << (64 - s);
    }
    return r;
}

static uint64_t hw_mod(const HostWide &a, uint64_t m)
{
    u128 rem = 0;
    for (int i = 3; i >= 0; --i) rem = ((rem << 64) | a.w[i]) % m;
    return (uint64_t)rem;
}

static double hw_to_double(const HostWide &a)
{
    double d = 0.0;
    for (int i = 3; i >= 0; --i) d = d * 18446744073709551616.0 + (double)a.w[i];
    return d;
}

struct Scaling {
    HostWide delta, half;
    double delta_inv;
};

// checks shared by decoding and encryption; max_limbs: what the caller can handle
static int scaling(int L, const uint64_t *moduli, int t_bits, Scaling *out)
{
    if (t_bits < 1 || t_bits > 32) return NIMBUS_COP_ERR_INVALID_ARG;
    for (int l = 0; l < L; ++l)
        if (moduli[l] <= (1ull << t_bits)) return NIMBUS_COP_ERR_INVALID_ARG;
    HostWide Q;
    Q.w[0] = 1;
    for (int l = 0; l < L; ++l) Q = hw_times(Q, moduli[l]);
    out->delta = hw_shift_right(Q, t_bits);
    out->half = hw_shift_right(out->delta, 1);
    out->delta_inv = 1.0 / hw_to_double(out->delta);
    return NIMBUS_COP_OK;
}

static hipError_t launch_secret(const RlweArgs &a, int logN, int L, const int8_t *s,
                                Twiddle *tables, hipStream_t stream)
{
    if (logN == 15) {
        return launch(rlwe_secret_kernel<15, 1>, dim3(2u * (unsigned)L), dim3(threads_for(14, 4)),
                      stream, a, s, tables);
    }
    NIMBUS_RLWE_DISPATCH(logN, launch(rlwe_secret_kernel<LOGN, 0>, dim3((unsigned)L),
                                      dim3(threads_for(LOGN, 4)), stream, a, s, tables));
}

}  // namespace nimbus

using namespace nimbus;

extern "C" {

size_t nimbus_rlwe_tables_bytes(int N, int L)
{
    if (N < (1 << kRlweMinLogN) || N > (1 << kRlweMaxLogN) || (N & (N - 1)) != 0) return 0;
    if (L < 1 || L > kMaxLimbs) return 0;
    return (size_t)L * limb_table_entries(N) * sizeof(Twiddle);
}

int nimbus_rlwe_setup(int N, int L, const uint64_t *moduli, const int8_t *s,
                      void *tables, size_t tables_bytes, void *stream)
{
    if (!s || !tables) return NIMBUS_COP_ERR_INVALID_ARG;
    RlweArgs a;
    const int rc = rlwe_check(N, L, moduli, &a);
    if (rc != NIMBUS_COP_OK) return rc;
    if (((uintptr_t)tables & 15u) != 0) return NIMBUS_COP_ERR_INVALID_ARG;
    if (tables_bytes < nimbus_rlwe_tables_bytes(N, L)) return NIMBUS_COP_ERR_BUFFER_SIZE;
    for (int l = 0; l < L; ++l) {
        const uint64_t q = moduli[l];
        uint64_t psi;
        if (!find_psi(q, N, &psi)) return NIMBUS_COP_ERR_INVALID_ARG;
        a.limb[l].psi = psi;
        a.limb[l].psi_inv = h_powmod(psi, 2ull * (uint64_t)N - 1, q);     // psi^(2N) = 1
        a.limb[l].n_inv = q - (q - 1) / (uint64_t)N;                      // N (q - (q-1)/N) = 1 mod q
    }
    const int logN = log2_exact(N);
    const unsigned total = (unsigned)N * (unsigned)L;
    if (launch(rlwe_powers_kernel, dim3((total + 255u) / 256u), dim3(256), (hipStream_t)stream,
               a, logN, L, (Twiddle *)tables) != hipSuccess)
        return NIMBUS_COP_ERR_LAUNCH;
    if (launch_secret(a, logN, L, s, (Twiddle *)tables, (hipStream_t)stream) != hipSuccess)
        return NIMBUS_COP_ERR_LAUNCH;
    // the same entries in the order of the product kernels: large batches, small batches
    const int pre = logN == 15 ? 1 : 0;
    const int maxs_of[kTableSets] = {0, logN == 15 ? 4 : stages_large_batch(logN),
                                     logN == 15 ? 4 : stages_small_batch(logN)};
    for (int set = 1; set < kTableSets; ++set) {
        if (launch(rlwe_table_set_kernel, dim3((total + 255u) / 256u), dim3(256), (hipStream_t)stream,
                   (Twiddle *)tables, logN, L, pre, maxs_of[set], set) != hipSuccess)
            return NIMBUS_COP_ERR_LAUNCH;
    }
    return NIMBUS_COP_OK;
}

int nimbus_rlwe_phase(const uint64_t *ct, int T, int N, int L, const uint64_t *moduli,
                      const void *tables, uint64_t *phi, void *stream)
{
    if (!ct || !tables || !phi || T < 0) return NIMBUS_COP_ERR_INVALID_ARG;
    PolyArgs a{};
    const int rc = rlwe_check(N, L, moduli, &a.limbs);
    if (rc != NIMBUS_COP_OK) return rc;
    if ((unsigned long long)T * (unsigned)L >= (1ull << 30)) return NIMBUS_COP_ERR_INVALID_ARG;
    if (T == 0) return NIMBUS_COP_OK;
    {
        const size_t poly_bytes = (size_t)L * (size_t)N * sizeof(uint64_t);
        if (ranges_overlap(phi, (size_t)T * poly_bytes, ct, 2u * (size_t)T * poly_bytes))
            return NIMBUS_COP_ERR_INVALID_ARG;
    }
    a.tables = (const Twiddle *)tables;
    a.L = L;
    a.src = ct;
    a.dst = phi;
    const hipError_t e = launch_poly<false>(a, log2_exact(N), (size_t)T * L, (hipStream_t)stream);
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

int nimbus_rlwe_decode(const uint64_t *phi, int T, int N, int L, const uint64_t *moduli,
                       int t_bits, uint64_t *m_hat, void *stream)
{
    if (!phi || !m_hat || T < 0) return NIMBUS_COP_ERR_INVALID_ARG;
    RlweArgs limbs;
    int rc = rlwe_check(N, L, moduli, &limbs);
    if (rc != NIMBUS_COP_OK) return rc;
    Scaling sc;
    rc = scaling(L, moduli, t_bits, &sc);
    if (rc != NIMBUS_COP_OK) return rc;
    const uint64_t total = (uint64_t)T * (uint64_t)N;
    if (total >= (1ull << 39)) return NIMBUS_COP_ERR_INVALID_ARG;
    // inverses of the Chinese remainder theorem; 0 = the moduli are not coprime
    uint64_t inv[kMaxLimbs][kMaxLimbs] = {};
    for (int j = 1; j < L; ++j)
        for (int i = 0; i < j; ++i) {
            inv[i][j] = h_invmod(moduli[i] % moduli[j], moduli[j]);
            if (inv[i][j] == 0) return NIMBUS_COP_ERR_INVALID_ARG;
        }
    if (T == 0) return NIMBUS_COP_OK;
    if (ranges_overlap(m_hat, (size_t)total * sizeof(uint64_t), phi, (size_t)total * (size_t)L * sizeof(uint64_t)))
        return NIMBUS_COP_ERR_INVALID_ARG;
    const dim3 grid((unsigned)((total + 255u) / 256u));
    hipError_t e;
    if (L <= 2) {
        DecodeArgs a{};
        a.phi = phi;
        a.m_hat = m_hat;
        a.L = L;
        a.logN = log2_exact(N);
        a.total = total;
        a.q0 = moduli[0];
        if (L == 2) {
            a.red1 = limbs.limb[1].red;
            a.q0_inv = inv[0][1];
        }
        a.delta_hi = sc.delta.w[1];
        a.delta_lo = sc.delta.w[0];
        a.half_hi = sc.half.w[1];
        a.half_lo = sc.half.w[0];
        a.delta_inv = sc.delta_inv;
        a.t_mask = (1ull << t_bits) - 1;
        e = launch(rlwe_decode_kernel, grid, dim3(256), (hipStream_t)stream, a);
    } else {
        DecodeWideArgs a{};
        a.phi = phi;
        a.m_hat = m_hat;
        a.L = L;
        a.logN = log2_exact(N);
        a.total = total;
        for (int l = 0; l < L; ++l) a.red[l] = limbs.limb[l].red;
        for (int i = 0; i < kMaxLimbs; ++i)
            for (int j = 0; j < kMaxLimbs; ++j) a.inv[i][j] = inv[i][j];
        for (int i = 0; i < 4; ++i) {
            a.delta.w[i] = sc.delta.w[i];
            a.half.w[i] = sc.half.w[i];
        }
        a.delta_inv = sc.delta_inv;
        a.t_mask = (1ull << t_bits) - 1;
        e = launch(rlwe_decode_wide_kernel, grid, dim3(256), (hipStream_t)stream, a);
    }
    return e == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

int nimbus_rlwe_decrypt(const uint64_t *ct, int T, int N, int L, const uint64_t *moduli,
                        int t_bits, const void *tables, uint64_t *phi, uint64_t *m_hat,
                        void *stream)
{
    if (!ct || !tables || !phi || !m_hat || T < 0) return NIMBUS_COP_ERR_INVALID_ARG;
    // every check of the second step before the first one is enqueued
    RlweArgs limbs;
    int rc = rlwe_check(N, L, moduli, &limbs);
    if (rc != NIMBUS_COP_OK) return rc;
    Scaling sc;
    rc = scaling(L, moduli, t_bits, &sc);
    if (rc != NIMBUS_COP_OK) return rc;
    if ((uint64_t)T * (uint64_t)N >= (1ull << 39)) return NIMBUS_COP_ERR_INVALID_ARG;
    for (int j = 1; j < L; ++j)
        for (int i = 0; i < j; ++i)
            if (h_invmod(moduli[i] % moduli[j], moduli[j]) == 0) return NIMBUS_COP_ERR_INVALID_ARG;
    {
        const size_t words = (size_t)T * (size_t)N;
        if (ranges_overlap(m_hat, words * sizeof(uint64_t), ct, 2u * words * (size_t)L * sizeof(uint64_t)) ||
            ranges_overlap(m_hat, words * sizeof(uint64_t), phi, words * (size_t)L * sizeof(uint64_t)))
            return NIMBUS_COP_ERR_INVALID_ARG;
    }
    rc = nimbus_rlwe_phase(ct, T, N, L, moduli, tables, phi, stream);
    if (rc != NIMBUS_COP_OK) return rc;
    return nimbus_rlwe_decode(phi, T, N, L, moduli, t_bits, m_hat, stream);
}

int nimbus_rlwe_encrypt(const uint64_t *W, int k, int n, int t_bits, int N, int L,
                        const uint64_t *moduli, const void *tables, const uint64_t *a_poly,
                        const int8_t *e, uint64_t *ctW, void *stream)
{
    if (!W || !tables || !a_poly || !e || !ctW) return NIMBUS_COP_ERR_INVALID_ARG;
    if (k < 1 || n < 1) return NIMBUS_COP_ERR_INVALID_ARG;
    PolyArgs a{};
    int rc = rlwe_check(N, L, moduli, &a.limbs);
    if (rc != NIMBUS_COP_OK) return rc;
    Scaling sc;
    rc = scaling(L, moduli, t_bits, &sc);
    if (rc != NIMBUS_COP_OK) return rc;
    const unsigned long long Ch = ((unsigned long long)n + (unsigned)N - 1) / (unsigned)N;
    const unsigned long long polys = (unsigned long long)k * Ch * (unsigned)L;
    if (polys >= (1ull << 30) || Ch * (unsigned)N >= (1ull << 31)) return NIMBUS_COP_ERR_INVALID_ARG;
    {
        const size_t rows = (size_t)k * (size_t)Ch;
        const size_t ct_bytes = rows * 2u * (size_t)L * (size_t)N * sizeof(uint64_t);
        if (ranges_overlap(ctW, ct_bytes, W, (size_t)k * (size_t)n * sizeof(uint64_t)) ||
            ranges_overlap(ctW, ct_bytes, a_poly, ct_bytes / 2) ||
            ranges_overlap(ctW, ct_bytes, e, rows * (size_t)N))
            return NIMBUS_COP_ERR_INVALID_ARG;
    }
    for (int l = 0; l < L; ++l) a.limbs.limb[l].delta = hw_mod(sc.delta, moduli[l]);
    a.tables = (const Twiddle *)tables;
    a.L = L;
    a.src = a_poly;
    a.dst = ctW;
    a.W = W;
    a.e = e;
    a.n = n;
    a.Ch = (int)Ch;
    const hipError_t err = launch_encrypt_rows(a, log2_exact(N), (size_t)polys, (hipStream_t)stream);
    return err == hipSuccess ? NIMBUS_COP_OK : NIMBUS_COP_ERR_LAUNCH;
}

}  // extern "C"
