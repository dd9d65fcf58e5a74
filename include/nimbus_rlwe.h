/*
 * nimbus_rlwe.h -- C ABI of the server side of the Nimbus linear layer on the GPU:
 * setup-phase row encoding + encryption of the weights, and decryption + decoding of the
 * ciphertexts the client sends back (arXiv 2411.15707).
 *
 * What the paper fixes and where:
 *   Setup (Algorithm 1, step 1; Section 3.2, Eq. (2)): the server encodes every row of W
 *   as one plaintext polynomial, w-hat_i[c] = W[i][c] for c in [n] and 0 elsewhere,
 *   encrypts it and sends the ciphertexts once; they are reused by every query.
 *   Online (Algorithm 1, step 5): the server decrypts the (masked, possibly packed)
 *   ciphertexts it receives; the result is its additive share of the layer output.
 *   Section 3.2 (complexity paragraph) notes that this decryption is the only place of
 *   the protocol that still pays a number-theoretic transform.
 *   Appendix B.1 names KeyGen / Enc / Dec over A_{N,q} = Z_q[X]/(X^N + 1) without printing
 *   formulas; this library uses the textbook coefficient-encoded symmetric scheme
 *       c1 = a,   c0 = -a s + e + Delta w-hat  (mod Q),   Delta = floor(Q / t),  t = 2^t_bits
 *       Dec:  phi = c0 + c1 s (mod Q),   m-hat[c] = floor((phi[c] + Delta/2) / Delta) mod t
 *   with Q = q_0 ... q_{L-1} held limb by limb (residue number system).
 *   For n > N (not covered by the paper) a row is cut into Ch = ceil(n/N) consecutive blocks
 *   of N columns, one polynomial each.
 *
 * The products a s and c1 s in Z_q[X]/(X^N + 1) are computed with a negacyclic
 * number-theoretic transform per limb (forward transform, pointwise product with the
 * transformed secret, inverse transform); results are exact residues, so any correct
 * method gives the same words.
 *
 * Randomness: the library draws none.  The uniform polynomials a and the small error
 * polynomials e are inputs of nimbus_rlwe_encrypt; the secret s is an input of
 * nimbus_rlwe_setup.
 *
 * Conventions (the same as nimbus_cop.h, whose status codes these functions return):
 *   - every pointer is a DEVICE pointer owned by the caller, except `moduli`, which is a
 *     HOST pointer to L primes, each odd, < 2^62 and = 1 modulo 2N (so that a primitive
 *     2N-th root of unity exists; a modulus without one is NIMBUS_COP_ERR_INVALID_ARG);
 *   - N is a power of two, 32 <= N <= 32768 (up to 16384 one polynomial is transformed
 *     inside the local memory of one compute unit, 32768 in two halves and a joining pass;
 *     N = 65536 is NIMBUS_COP_ERR_UNSUPPORTED);
 *   - 1 <= L <= 4 distinct primes (Q < 2^248); 1 <= t_bits <= 32 and 2^t_bits < q_l for
 *     decoding and encryption;
 *   - nothing is allocated, freed or synchronised; all work is enqueued on `stream`
 *     (a hipStream_t, NULL = the default stream); on any error nothing is enqueued;
 *   - a buffer that is written must not overlap a buffer that is read (checked on the host from
 *     the sizes: NIMBUS_COP_ERR_INVALID_ARG);
 *   - residues handed in must be canonical (in [0, q_l)); residues written are canonical;
 *   - re-entrant; concurrent calls on different streams are allowed as long as their
 *     outputs do not overlap.
 */
#ifndef NIMBUS_RLWE_H
#define NIMBUS_RLWE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Size in bytes of the per-key table buffer for ring degree N and L limbs (transform
 * constants and the transformed secret, per limb, three times over: in their natural order and
 * in the two orders in which the kernels for large and for small batches read them;
 * 144 N L bytes); 0 for arguments out of range. */
size_t nimbus_rlwe_tables_bytes(int N, int L);

/* KeyGen side of Appendix B.1, once per secret key: fills `tables` (at least
 * nimbus_rlwe_tables_bytes(N, L) bytes, 16-byte aligned) with, per limb, the powers of a
 * primitive 2N-th root of unity used by the forward and inverse negacyclic transforms and
 * the transform of the secret s.
 *   s       [N] int8, small signed coefficients (ternary in this build's harness); a
 *           negative coefficient stands for q_l minus its magnitude
 *   tables  written; read-only afterwards, shared by every later call with the same
 *           (N, L, moduli, s)
 * Errors: INVALID_ARG (null pointer, N / L / modulus out of range, no 2N-th root of unity
 * found), UNSUPPORTED (N > 32768), BUFFER_SIZE (tables_bytes too small), LAUNCH. */
int nimbus_rlwe_setup(int N, int L, const uint64_t *moduli, const int8_t *s,
                      void *tables, size_t tables_bytes, void *stream);

/* Phase of T ciphertexts, per limb (the first half of Dec, Appendix B.1):
 *   phi[r][l][.] = ct[r][0][l][.] + ct[r][1][l][.] * s   in Z_{q_l}[X]/(X^N + 1).
 *   ct   [T][2][L][N] canonical residues, polynomial 0 = c0, 1 = c1, coefficient order
 *   phi  [T][L][N], written, canonical residues; must not overlap ct
 * T = 0 is a no-op.  Any L in [1, 4]. */
int nimbus_rlwe_phase(const uint64_t *ct, int T, int N, int L, const uint64_t *moduli,
                      const void *tables, uint64_t *phi, void *stream);

/* Decoding of T phases (the second half of Dec): the limb phases are combined by the
 * Chinese remainder theorem into phi in [0, Q), then
 *   m_hat[r][c] = floor((phi[r][c] + floor(Delta/2)) / Delta) mod 2^t_bits,  Delta = floor(Q / 2^t_bits).
 *   phi    [T][L][N] canonical residues
 *   m_hat  [T][N], written, values < 2^t_bits */
int nimbus_rlwe_decode(const uint64_t *phi, int T, int N, int L, const uint64_t *moduli,
                       int t_bits, uint64_t *m_hat, void *stream);

/* Dec of Appendix B.1 / Algorithm 1 step 5: nimbus_rlwe_phase followed by
 * nimbus_rlwe_decode on the same stream.
 *   phi    [T][L][N] workspace, written (the phases, useful for measuring the noise)
 *   m_hat  [T][N], written */
int nimbus_rlwe_decrypt(const uint64_t *ct, int T, int N, int L, const uint64_t *moduli,
                        int t_bits, const void *tables, uint64_t *phi, uint64_t *m_hat,
                        void *stream);

/* Setup phase of Algorithm 1 (step 1): row-wise encoding of W (Section 3.2, Eq. (2), with
 * the chunking for n > N) fused with the encryption of every row.
 *   W    [k][n] row-major, every entry < 2^t_bits
 *   a    [k][Ch][L][N] canonical residues: the uniform polynomial of each ciphertext
 *   e    [k][Ch][N] int8: the error polynomial of each ciphertext
 *   ctW  [k][Ch][2][L][N], written: the layout nimbus_cop_matmul / nimbus_cop_prepare read;
 *        ctW[i][ch][1] = a[i][ch],
 *        ctW[i][ch][0][l] = (Delta mod q_l) * w-hat_{i,ch} + e[i][ch] - a[i][ch][l] * s  (mod q_l)
 *        must not overlap the inputs
 * k >= 1, n >= 1. */
int nimbus_rlwe_encrypt(const uint64_t *W, int k, int n, int t_bits, int N, int L,
                        const uint64_t *moduli, const void *tables, const uint64_t *a,
                        const int8_t *e, uint64_t *ctW, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NIMBUS_RLWE_H */
