/*
 * CPU oracle for the Client-side Outer Product (COP) linear layer of Nimbus
 * (arXiv 2411.15707).  TEST INFRASTRUCTURE ONLY: this file is what the HIP
 * library is checked against.  It shares no code with the HIP path and must
 * never be called from it; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg load it.
 *
 * Everything here is the plain definition, written for checking by eye against
 * the paper: 128-bit integers, one loop per index, no blocking, no lazy
 * reduction tricks.
 *
 * Dimension names (the paper's letters in brackets):
 *   m  tokens, rows of the client's share matrix X            [k]
 *   k  inner dimension, rows of W = number of weight ciphertexts [m]
 *   n  output features, columns of W                            [n]
 *   N  ring degree, L RNS limbs q_0..q_{L-1}, Q = prod q_l, t = 2^t_bits.
 *
 * Canonical ciphertext layout used everywhere:  [row][Ch][2][L][N]
 *   Ch = ceil(n/N) ring chunks, polynomial 0 = b-hat (c0), 1 = a-hat (c1).
 *
 * Parity pins (tests/test_oracle_*.py): Python big-int recomputation, special
 * cases (X = 0, X = identity, k = 1, all-ones), numpy object matmul, the
 * decryption invariant Dec(out_j) + R_j = (X W)_j mod t with a brute-force
 * right-hand side, enc/dec round trip, additive and scalar homomorphism,
 * negacyclic X^N = -1, Table 5 size accounting; for shares of up to 64 bits:
 * big-int recomputation, agreement with the narrow version, the high/low half
 * identity, phase linearity; for the right-shift packing:
 * RShift against the dense negacyclic product by X^s, N unit shifts = negation,
 * P = 1 is the identity, and the decryption invariant on packed ciphertexts.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef unsigned __int128 u128;
typedef __int128 i128;

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * COP accumulation + masking.
 * Algorithm 1 step 2:  c[j] = (+)_{i in [k]}  X[j][i] (x) [[W_i]]
 *   with (x) = scalar times both ciphertext polynomials, coefficient-wise
 *   mod q, and (+) = coefficient-wise addition mod q (Appendix B.1).
 * Algorithm 1 step 4 (arithmetic only): add the caller's mask polynomial pair.
 * Every RNS limb is an independent column with its own modulus.
 * All N coefficients of every chunk are computed: after encryption the padding
 * positions n..N-1 are as dense as the rest.
 * mask may be NULL (= no mask).  Returns the number of threads used.
 * ---------------------------------------------------------------------- */
int oracle_cop_ref(const uint64_t *X, int m, int k,
                   const uint64_t *ctW, int n, int N, int L,
                   const uint64_t *moduli,
                   const uint64_t *mask, uint64_t *out, int threads)
{
    const int Ch = (n + N - 1) / N;
    const size_t C = (size_t)Ch * 2 * L * N;     /* residues per ciphertext row */
    int used = 1;
    if (threads < 1) threads = 1;
#pragma omp parallel num_threads(threads)
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        /* exact integer accumulator of one output ciphertext row; the sum of
         * k products of a <= 32-bit share and a < 2^62 residue stays far
         * below 2^128 */
        u128 *acc = (u128 *)malloc(sizeof(u128) * C);
#pragma omp for schedule(static)
        for (int j = 0; j < m; ++j) {                    /* output row = token j */
            for (size_t col = 0; col < C; ++col) acc[col] = 0;
            for (int i = 0; i < k; ++i) {                /* weight row i */
                const uint64_t x = X[(size_t)j * k + i]; /* scalar x_{j,i} */
                const uint64_t *ct = ctW + (size_t)i * C;
                for (size_t col = 0; col < C; ++col)     /* (x) then (+) */
                    acc[col] += (u128)x * ct[col];
            }
            for (size_t col = 0; col < C; ++col) {
                const int l = (int)((col / N) % L);      /* [Ch][2][L][N] -> limb */
                u128 v = acc[col];
                if (mask) v += mask[(size_t)j * C + col];
                out[(size_t)j * C + col] = (uint64_t)(v % moduli[l]);
            }
        }
        free(acc);
    }
    return used;
}

/* ------------------------------------------------------------------------
 * The same for shares of up to 64 bits (the paper's own parameter set uses
 * l = 64, Section 5.1 "Experimental setup"): a product of a 64-bit share and
 * a < 2^62 residue still fits 128 bits, a sum of them does not, so every
 * product is reduced before it is added:
 *   acc = (acc + (x * c mod q_l)) , acc < k * q_l  < 2^86
 * ---------------------------------------------------------------------- */
int oracle_cop_ref_wide(const uint64_t *X, int m, int k,
                        const uint64_t *ctW, int n, int N, int L,
                        const uint64_t *moduli,
                        const uint64_t *mask, uint64_t *out, int threads)
{
    const int Ch = (n + N - 1) / N;
    const size_t C = (size_t)Ch * 2 * L * N;
    int used = 1;
    if (threads < 1) threads = 1;
#pragma omp parallel num_threads(threads)
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        u128 *acc = (u128 *)malloc(sizeof(u128) * C);
#pragma omp for schedule(static)
        for (int j = 0; j < m; ++j) {
            for (size_t col = 0; col < C; ++col) acc[col] = 0;
            for (int i = 0; i < k; ++i) {
                const uint64_t x = X[(size_t)j * k + i];
                const uint64_t *ct = ctW + (size_t)i * C;
                for (size_t col = 0; col < C; ++col) {
                    const uint64_t q = moduli[(col / N) % L];
                    acc[col] += ((u128)x * ct[col]) % q;
                }
            }
            for (size_t col = 0; col < C; ++col) {
                const int l = (int)((col / N) % L);
                u128 v = acc[col];
                if (mask) v += mask[(size_t)j * C + col];
                out[(size_t)j * C + col] = (uint64_t)(v % moduli[l]);
            }
        }
        free(acc);
    }
    return used;
}

/* ------------------------------------------------------------------------
 * Row-wise encoding, Eq. (2):  w-hat_i[c] = W[i][c] for c in [n], rest zero.
 * For n > N (not covered by the paper) the columns are cut into Ch consecutive
 * blocks of N; block ch of row i becomes its own polynomial.
 * W is [k][n], w_hat is [k][Ch][N].
 * ---------------------------------------------------------------------- */
void oracle_encode_rows(const uint64_t *W, int k, int n, int N, uint64_t *w_hat)
{
    const int Ch = (n + N - 1) / N;
    for (int i = 0; i < k; ++i)
        for (int ch = 0; ch < Ch; ++ch)
            for (int c = 0; c < N; ++c) {
                const long col = (long)ch * N + c;
                w_hat[((size_t)i * Ch + ch) * N + c] = col < n ? W[(size_t)i * n + col] : 0;
            }
}

/* ------------------------------------------------------------------------
 * Negacyclic product in Z_q[X]/(X^N+1) of a (residues) by a polynomial s with
 * small signed coefficients (the ternary secret):
 *   out[c] = sum_{j<=c} a[j] s[c-j]  -  sum_{j>c} a[j] s[N+c-j]   (mod q)
 * Schoolbook, O(N^2); the wrapped terms change sign because X^N = -1.
 * ---------------------------------------------------------------------- */
void oracle_negacyclic_mul_small(const uint64_t *a, const int8_t *s, int N,
                                 uint64_t q, uint64_t *out)
{
    for (int c = 0; c < N; ++c) {
        i128 acc = 0;
        for (int j = 0; j < N; ++j) {
            const int d = c - j;
            if (d >= 0) acc += (i128)a[j] * s[d];
            else        acc -= (i128)a[j] * s[N + d];
        }
        i128 r = acc % (i128)q;
        if (r < 0) r += q;
        out[c] = (uint64_t)r;
    }
}

static u128 big_Q(const uint64_t *moduli, int L)
{
    u128 Q = 1;
    for (int l = 0; l < L; ++l) Q *= moduli[l];
    return Q;
}

/* ------------------------------------------------------------------------
 * Symmetric-key RLWE encryption of `rows` plaintext polynomials (Appendix B.1
 * names Enc but prints no formula; this is the textbook coefficient-encoded
 * scheme the build's parameters assume):
 *     c1 = a,   c0 = -a s + e + Delta * w_hat   (mod Q),   Delta = floor(Q/t)
 * stored limb by limb.  Since Delta * w_hat < Q, its residue mod q_l is
 * (Delta mod q_l) * w_hat mod q_l.
 *   w_hat [rows][N] values < t;  s [N] in {-1,0,1};  a [rows][L][N] residues;
 *   e [rows][N] small signed;  ct out [rows][2][L][N].
 * Requires L <= 2 so that Q fits 128 bits.  Returns 0, or -1 if L > 2.
 * ---------------------------------------------------------------------- */
int oracle_encrypt(const uint64_t *w_hat, int rows, const int8_t *s,
                   const uint64_t *a, const int8_t *e,
                   int N, int L, const uint64_t *moduli, int t_bits,
                   uint64_t *ct, int threads)
{
    if (L > 2) return -1;
    const u128 Q = big_Q(moduli, L);
    const u128 Delta = Q >> t_bits;              /* floor(Q / 2^t_bits) */
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
    for (int r = 0; r < rows; ++r) {
        uint64_t *as = (uint64_t *)malloc(sizeof(uint64_t) * N);
        for (int l = 0; l < L; ++l) {
            const uint64_t q = moduli[l];
            const uint64_t dl = (uint64_t)(Delta % q);
            const uint64_t *al = a + ((size_t)r * L + l) * N;
            uint64_t *c0 = ct + (((size_t)r * 2 + 0) * L + l) * N;
            uint64_t *c1 = ct + (((size_t)r * 2 + 1) * L + l) * N;
            oracle_negacyclic_mul_small(al, s, N, q, as);
            for (int c = 0; c < N; ++c) {
                i128 v = (i128)((u128)dl * w_hat[(size_t)r * N + c] % q);
                v += e[(size_t)r * N + c];
                v -= as[c];
                v %= (i128)q;
                if (v < 0) v += q;
                c0[c] = (uint64_t)v;
                c1[c] = al[c];
            }
        }
        free(as);
    }
    return 0;
}

/* phase of one ciphertext, per limb:  phi_l = c0_l + c1_l * s  (mod q_l).
 * ct is [2][L][N]; phi is [L][N]. */
void oracle_phase(const uint64_t *ct, const int8_t *s, int N, int L,
                  const uint64_t *moduli, uint64_t *phi)
{
    uint64_t *as = (uint64_t *)malloc(sizeof(uint64_t) * N);
    for (int l = 0; l < L; ++l) {
        const uint64_t q = moduli[l];
        const uint64_t *c0 = ct + ((size_t)0 * L + l) * N;
        const uint64_t *c1 = ct + ((size_t)1 * L + l) * N;
        oracle_negacyclic_mul_small(c1, s, N, q, as);
        for (int c = 0; c < N; ++c)
            phi[(size_t)l * N + c] = (uint64_t)(((u128)c0[c] + as[c]) % q);
    }
    free(as);
}

/* modular inverse by the extended Euclid algorithm, a and mod coprime */
static uint64_t inv_mod(uint64_t a, uint64_t mod)
{
    i128 r0 = mod, r1 = a % mod, t0 = 0, t1 = 1;
    while (r1 != 0) {
        i128 qq = r0 / r1;
        i128 r2 = r0 - qq * r1; r0 = r1; r1 = r2;
        i128 t2 = t0 - qq * t1; t0 = t1; t1 = t2;
    }
    if (t0 < 0) t0 += mod;
    return (uint64_t)t0;
}

/* ------------------------------------------------------------------------
 * Decryption + decoding of one ciphertext [2][L][N]:
 *   phi = c0 + c1 s mod Q (CRT of the limb phases, Garner's formula for L=2),
 *   m_hat[c] = floor((phi[c] + Delta/2) / Delta) mod t.
 * Also returns, if noise != NULL, the centred noise  phi - Delta*m_hat  lifted
 * to (-Q/2, Q/2] and saturated to int64.
 * Requires L <= 2.  Returns 0 or -1.
 * ---------------------------------------------------------------------- */
int oracle_decrypt(const uint64_t *ct, const int8_t *s, int N, int L,
                   const uint64_t *moduli, int t_bits,
                   uint64_t *m_hat, int64_t *noise)
{
    if (L > 2) return -1;
    const u128 Q = big_Q(moduli, L);
    const u128 Delta = Q >> t_bits;
    const uint64_t tmask = ((uint64_t)1 << t_bits) - 1;
    uint64_t *phi = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)L * N);
    oracle_phase(ct, s, N, L, moduli, phi);
    uint64_t q0inv = 0;
    if (L == 2) q0inv = inv_mod(moduli[0] % moduli[1], moduli[1]);
    for (int c = 0; c < N; ++c) {
        u128 v = phi[c];
        if (L == 2) {
            /* v = p0 + q0 * ((p1 - p0) * q0^{-1} mod q1) */
            const uint64_t q1 = moduli[1];
            const uint64_t p0 = phi[c] % q1, p1 = phi[(size_t)N + c];
            const uint64_t diff = (uint64_t)(((u128)p1 + q1 - p0) % q1);
            const uint64_t h = (uint64_t)((u128)diff * q0inv % q1);
            v = (u128)phi[c] + (u128)moduli[0] * h;
        }
        const u128 mm = (v + Delta / 2) / Delta;
        m_hat[c] = (uint64_t)mm & tmask;
        if (noise) {
            /* v - Delta*m_hat, taken modulo Q into (-Q/2, Q/2] */
            i128 d = (i128)v - (i128)(Delta * (u128)m_hat[c]);
            if (d > (i128)(Q / 2)) d -= (i128)Q;
            if (d < -(i128)(Q / 2)) d += (i128)Q;
            if (d > INT64_MAX) d = INT64_MAX;
            if (d < INT64_MIN) d = INT64_MIN;
            noise[c] = (int64_t)d;
        }
    }
    free(phi);
    return 0;
}

/* ------------------------------------------------------------------------
 * Mask polynomial pair that realises "subtract the client's output share R"
 * (Algorithm 1 step 4) as an addition:  c0 part = (Q - Delta * R[c]) mod Q per
 * limb, c1 part = 0.   R is [N] values < t, mask is [2][L][N].  L <= 2.
 * ---------------------------------------------------------------------- */
int oracle_share_mask(const uint64_t *R, int N, int L, const uint64_t *moduli,
                      int t_bits, uint64_t *mask)
{
    if (L > 2) return -1;
    const u128 Q = big_Q(moduli, L);
    const u128 Delta = Q >> t_bits;
    for (int l = 0; l < L; ++l) {
        const uint64_t q = moduli[l];
        for (int c = 0; c < N; ++c) {
            const u128 v = (Q - Delta * R[c]) % Q;
            mask[((size_t)0 * L + l) * N + c] = (uint64_t)(v % q);
            mask[((size_t)1 * L + l) * N + c] = 0;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Right shift (Appendix B.1): RShift(ct, s) multiplies both polynomials of a
 * ciphertext by the monomial X^s in Z_q[X]/(X^N+1), 0 <= s < N: coefficient c
 * moves to c+s, and a coefficient that passes the end re-enters at c+s-N with
 * its sign flipped (X^N = -1).  ct and out are [2][L][N]; out must not alias ct.
 * ---------------------------------------------------------------------- */
void oracle_rshift(const uint64_t *ct, int s, int N, int L, const uint64_t *moduli, uint64_t *out)
{
    for (int p = 0; p < 2; ++p)
        for (int l = 0; l < L; ++l) {
            const uint64_t q = moduli[l];
            const uint64_t *src = ct + ((size_t)p * L + l) * N;
            uint64_t *dst = out + ((size_t)p * L + l) * N;
            for (int c = 0; c < N; ++c) {
                const int to = c + s;
                if (to < N) dst[to] = src[c];
                else        dst[to - N] = src[c] == 0 ? 0 : q - src[c];
            }
        }
}

/* ------------------------------------------------------------------------
 * Output packing, Algorithm 1 step 3 (n <= N, one ring chunk): with
 * P = floor(N/n) rows per packed ciphertext,
 *   packed[theta] = (+)_{u in [P]}  RShift(rows[theta*P + u], u*n)   (+) mask[theta]
 * for theta in [ceil(m/P)]; rows past m count as zero ciphertexts.  The shift
 * amounts are multiples of n (the printed algorithm writes another letter; the
 * figure shifts the second ciphertext by the width of the first one's payload).
 * rows is [m][2][L][N], mask is [ceil(m/P)][2][L][N] or NULL, packed likewise.
 * Returns the number of packed ciphertexts, or -1 if n > N.
 * ---------------------------------------------------------------------- */
int oracle_pack_ref(const uint64_t *rows, int m, int n, int N, int L, const uint64_t *moduli,
                    const uint64_t *mask, uint64_t *packed)
{
    if (n > N || n <= 0) return -1;
    const int P = N / n;
    const int T = (m + P - 1) / P;
    const size_t ct_words = (size_t)2 * L * N;
    uint64_t *tmp = (uint64_t *)malloc(ct_words * sizeof(uint64_t));
    if (!tmp) return -1;
    for (int th = 0; th < T; ++th) {
        uint64_t *dst = packed + (size_t)th * ct_words;
        memset(dst, 0, ct_words * sizeof(uint64_t));
        for (int u = 0; u < P; ++u) {
            const int j = th * P + u;
            if (j >= m) break;
            oracle_rshift(rows + (size_t)j * ct_words, u * n, N, L, moduli, tmp);
            for (int p = 0; p < 2; ++p)
                for (int l = 0; l < L; ++l) {
                    const uint64_t q = moduli[l];
                    for (int c = 0; c < N; ++c) {
                        const size_t at = ((size_t)p * L + l) * N + c;
                        dst[at] = (uint64_t)(((u128)dst[at] + tmp[at]) % q);
                    }
                }
        }
        if (mask)
            for (int p = 0; p < 2; ++p)
                for (int l = 0; l < L; ++l) {
                    const uint64_t q = moduli[l];
                    for (int c = 0; c < N; ++c) {
                        const size_t at = ((size_t)p * L + l) * N + c;
                        dst[at] = (uint64_t)(((u128)dst[at] + mask[(size_t)th * ct_words + at]) % q);
                    }
                }
    }
    free(tmp);
    return T;
}

/* ========================================================================
 * The same scheme for up to four limbs (Q up to 2^248): 256-bit integers as
 * four 64-bit words, least significant first, with the schoolbook routines
 * below (add, subtract, compare, times a word, shift right, remainder by a
 * word, and bit-by-bit long division).  Slow and plain on purpose.
 * Pins (tests/test_oracle_rns.py): agreement with oracle_encrypt /
 * oracle_decrypt for one and two limbs, Python integers for three and four
 * limbs (reconstructed value congruent to every limb phase and below Q,
 * rounding division at and next to its boundaries), enc/dec round trip.
 * ====================================================================== */
typedef struct { uint64_t w[4]; } u256;

static u256 u256_from_u64(uint64_t v)
{
    u256 r = {{v, 0, 0, 0}};
    return r;
}

static int u256_cmp(const u256 *a, const u256 *b)
{
    for (int i = 3; i >= 0; --i) {
        if (a->w[i] < b->w[i]) return -1;
        if (a->w[i] > b->w[i]) return 1;
    }
    return 0;
}

static u256 u256_add(const u256 *a, const u256 *b)
{
    u256 r;
    u128 carry = 0;
    for (int i = 0; i < 4; ++i) {
        const u128 s = (u128)a->w[i] + b->w[i] + carry;
        r.w[i] = (uint64_t)s;
        carry = s >> 64;
    }
    return r;
}

static u256 u256_sub(const u256 *a, const u256 *b)      /* a >= b */
{
    u256 r;
    uint64_t borrow = 0;
    for (int i = 0; i < 4; ++i) {
        const u128 d = (u128)a->w[i] - b->w[i] - borrow;
        r.w[i] = (uint64_t)d;
        borrow = (uint64_t)(d >> 64) & 1u;
    }
    return r;
}

static u256 u256_mul_u64(const u256 *a, uint64_t m)     /* product must fit 256 bits */
{
    u256 r;
    u128 carry = 0;
    for (int i = 0; i < 4; ++i) {
        const u128 p = (u128)a->w[i] * m + carry;
        r.w[i] = (uint64_t)p;
        carry = p >> 64;
    }
    return r;
}

static u256 u256_shr(const u256 *a, int s)              /* 0 <= s < 256 */
{
    u256 r = {{0, 0, 0, 0}};
    const int ws = s / 64, bs = s % 64;
    for (int i = 0; i + ws < 4; ++i) {
        uint64_t v = a->w[i + ws] >> bs;
        if (bs && i + ws + 1 < 4) v |= a->w[i + ws + 1] << (64 - bs);
        r.w[i] = v;
    }
    return r;
}

static uint64_t u256_mod_u64(const u256 *a, uint64_t m)
{
    u128 rem = 0;
    for (int i = 3; i >= 0; --i) rem = ((rem << 64) | a->w[i]) % m;
    return (uint64_t)rem;
}

static int u256_bit(const u256 *a, int i) { return (int)((a->w[i / 64] >> (i % 64)) & 1u); }

/* quotient of a by d (d > 0), bit by bit from the top */
static u256 u256_div(const u256 *a, const u256 *d)
{
    u256 quo = {{0, 0, 0, 0}}, rem = {{0, 0, 0, 0}};
    for (int i = 255; i >= 0; --i) {
        /* rem = 2 rem + bit i of a   (rem < d <= 2^255 would be needed for the shift not
         * to overflow; Q < 2^248 keeps every value here far below that) */
        const u256 twice = u256_add(&rem, &rem);
        rem = twice;
        rem.w[0] |= (uint64_t)u256_bit(a, i);
        if (u256_cmp(&rem, d) >= 0) {
            rem = u256_sub(&rem, d);
            quo.w[i / 64] |= (uint64_t)1 << (i % 64);
        }
    }
    return quo;
}

static u256 rns_Q(const uint64_t *moduli, int L)
{
    u256 Q = u256_from_u64(1);
    for (int l = 0; l < L; ++l) Q = u256_mul_u64(&Q, moduli[l]);
    return Q;
}

/* ------------------------------------------------------------------------
 * Encryption as oracle_encrypt, for 1 <= L <= 4:
 *     c1 = a,   c0 = -a s + e + Delta * w_hat  (mod Q),   Delta = floor(Q / 2^t_bits),
 * limb by limb with (Delta mod q_l).  Shapes as oracle_encrypt.  Returns 0, or -1 for L
 * out of range.
 * ---------------------------------------------------------------------- */
int oracle_encrypt_rns(const uint64_t *w_hat, int rows, const int8_t *s,
                       const uint64_t *a, const int8_t *e,
                       int N, int L, const uint64_t *moduli, int t_bits,
                       uint64_t *ct, int threads)
{
    if (L < 1 || L > 4) return -1;
    const u256 Q = rns_Q(moduli, L);
    const u256 Delta = u256_shr(&Q, t_bits);
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1)
    for (int r = 0; r < rows; ++r) {
        uint64_t *as = (uint64_t *)malloc(sizeof(uint64_t) * N);
        for (int l = 0; l < L; ++l) {
            const uint64_t q = moduli[l];
            const uint64_t dl = u256_mod_u64(&Delta, q);
            const uint64_t *al = a + ((size_t)r * L + l) * N;
            uint64_t *c0 = ct + (((size_t)r * 2 + 0) * L + l) * N;
            uint64_t *c1 = ct + (((size_t)r * 2 + 1) * L + l) * N;
            oracle_negacyclic_mul_small(al, s, N, q, as);
            for (int c = 0; c < N; ++c) {
                i128 v = (i128)((u128)dl * w_hat[(size_t)r * N + c] % q);
                v += e[(size_t)r * N + c];
                v -= as[c];
                v %= (i128)q;
                if (v < 0) v += q;
                c0[c] = (uint64_t)v;
                c1[c] = al[c];
            }
        }
        free(as);
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Decryption + decoding of one ciphertext [2][L][N] for 1 <= L <= 4:
 *   phase per limb, then the unique phi in [0, Q) with phi = phi_l (mod q_l) for every l
 *   (Chinese remainder theorem, built limb by limb: if v is right modulo q_0 .. q_{j-1},
 *   whose product is M, then v + M * ((phi_j - v) * M^-1 mod q_j) is right modulo q_j as
 *   well), then  m_hat[c] = floor((phi[c] + floor(Delta/2)) / Delta) mod 2^t_bits.
 * Returns 0, or -1 for L out of range.
 * ---------------------------------------------------------------------- */
int oracle_decrypt_rns(const uint64_t *ct, const int8_t *s, int N, int L,
                       const uint64_t *moduli, int t_bits, uint64_t *m_hat)
{
    if (L < 1 || L > 4) return -1;
    const u256 Q = rns_Q(moduli, L);
    const u256 Delta = u256_shr(&Q, t_bits);
    const u256 half = u256_shr(&Delta, 1);
    const uint64_t tmask = t_bits >= 64 ? ~(uint64_t)0 : (((uint64_t)1 << t_bits) - 1);
    uint64_t *phi = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)L * N);
    oracle_phase(ct, s, N, L, moduli, phi);
    for (int c = 0; c < N; ++c) {
        u256 v = u256_from_u64(phi[c]);
        u256 M = u256_from_u64(moduli[0]);
        for (int j = 1; j < L; ++j) {
            const uint64_t qj = moduli[j];
            const uint64_t vj = u256_mod_u64(&v, qj);
            const uint64_t Mj = u256_mod_u64(&M, qj);
            const uint64_t diff = (uint64_t)(((u128)phi[(size_t)j * N + c] + qj - vj) % qj);
            const uint64_t h = (uint64_t)((u128)diff * inv_mod(Mj, qj) % qj);
            const u256 step = u256_mul_u64(&M, h);
            v = u256_add(&v, &step);
            M = u256_mul_u64(&M, qj);
        }
        const u256 num = u256_add(&v, &half);
        const u256 mm = u256_div(&num, &Delta);
        m_hat[c] = mm.w[0] & tmask;
    }
    free(phi);
    return 0;
}

/* Mask polynomial pair of oracle_share_mask for 1 <= L <= 4:
 * c0 part = (Q - Delta * R[c]) mod Q per limb, c1 part = 0. */
int oracle_share_mask_rns(const uint64_t *R, int N, int L, const uint64_t *moduli,
                          int t_bits, uint64_t *mask)
{
    if (L < 1 || L > 4) return -1;
    const u256 Q = rns_Q(moduli, L);
    const u256 Delta = u256_shr(&Q, t_bits);
    for (int c = 0; c < N; ++c) {
        const u256 dr = u256_mul_u64(&Delta, R[c]);          /* <= Delta * (t - 1) < Q */
        u256 v = u256_sub(&Q, &dr);
        if (u256_cmp(&v, &Q) >= 0) v = u256_sub(&v, &Q);     /* R[c] = 0 */
        for (int l = 0; l < L; ++l) {
            mask[((size_t)0 * L + l) * N + c] = u256_mod_u64(&v, moduli[l]);
            mask[((size_t)1 * L + l) * N + c] = 0;
        }
    }
    return 0;
}
