/*
 * nimbus_cop.h -- C ABI of the MI355X (gfx950) library for the client side of
 * the Client-side Outer Product (COP) linear layer of Nimbus (arXiv 2411.15707).
 *
 * What one call computes (Algorithm 1, step 2 and the arithmetic of step 4;
 * the homomorphic operations (x) and (+) of Appendix B.1):
 *
 *     out[j] = ( (+)_{i in [k]}  X[j][i] (x) [[W_i]] )  (+)  mask[j]      j in [m]
 *
 * i.e. for every RNS limb l, both ciphertext polynomials p and every
 * coefficient c of every ring chunk ch
 *
 *     out[j][ch][p][l][c] = ( sum_i X[j][i] * ctW[i][ch][p][l][c]
 *                             + mask[j][ch][p][l][c] )  mod q_l ,
 *
 * written as the canonical residue in [0, q_l).  The result is exact; there is
 * exactly one correct bit pattern.
 *
 * Dimension names (the paper's letters in brackets):
 *   m  tokens = rows of the client's share matrix X = output ciphertexts   [k]
 *   k  inner dimension = rows of W = number of weight ciphertexts          [m]
 *   n  output features = used coefficients (row-wise encoding, Eq. (2))    [n]
 *   N  ring degree, L RNS limbs, Ch = ceil(n / N) ring chunks (the paper
 *      assumes n <= N; for n > N each weight row is Ch ciphertexts, chunk ch
 *      holding columns ch*N .. ch*N+N-1 of W).
 *
 * Canonical ciphertext layout, row-major:  [row][Ch][2][L][N]  of uint64_t,
 * polynomial 0 = b-hat, 1 = a-hat.  All N coefficients are processed: after
 * encryption the positions n..N-1 are as dense as the others.
 *
 * Memory: X, ctW, mask, out, prepared and workspace are DEVICE pointers owned by
 * the caller; `moduli` is a HOST pointer read during the call.  The library
 * never allocates, frees or synchronises: work is enqueued on `stream`
 * (a hipStream_t; NULL = the default stream) and the call returns at once.
 * `out` (and `workspace`, `prepared`, `packed` where they are written) must not overlap any
 * other buffer of the call: checked on the host from the sizes, NIMBUS_COP_ERR_INVALID_ARG.
 * Calls are re-entrant; calls that share a
 * workspace must be ordered on one stream.
 *
 * Preconditions on device data (not checked): X[j][i] < 2^x_bits,
 * residues of ctW and mask < q_l.
 *
 * Errors: every function returning int gives NIMBUS_COP_OK (0) or a negative
 * code.  Every code but NIMBUS_COP_ERR_LAUNCH is found on the host before
 * anything is enqueued: `out` is untouched.  NIMBUS_COP_ERR_LAUNCH means that
 * the HIP runtime refused a kernel launch; an entry point that launches more
 * than one kernel (nimbus_cop_matmul_prepared and its _static variant,
 * nimbus_cop_prepare, nimbus_cop_check_inputs, and the staged entry points
 * for shares of more than 32 bits) may then already have enqueued the earlier
 * ones, and what its outputs and workspace hold is unspecified.  No C++
 * exception crosses this boundary.
 *
 * Loading: the library links the HIP runtime (libamdhip64) by name.  A process
 * must map ONE copy of that runtime: device pointers and streams made by one
 * copy mean nothing to another, and the first launch fails.  A host program
 * that brings its own copy (PyTorch loads the one in its wheel by path) has to
 * load it BEFORE this library, so that the dynamic linker resolves this
 * library's dependency to the copy already mapped; the Python binding imports
 * torch first for that reason.
 *
 * Accepted parameters: m, k, n >= 1; N a power of two in [32, 65536];
 * L in [1, 4]; x_bits in [1, 32] with every q_l odd and 2^x_bits < q_l < 2^62;
 * k < 2^24; m <= 2^30; Ch*2*L*N < 2^31.
 * Shares of 33 to 64 bits (the paper's own setting is l = 64, Section 5.1
 * "Experimental setup") are accepted by the prepared-weights entry points only
 * (nimbus_cop_workspace_bytes, nimbus_cop_stage_shares, nimbus_cop_matmul_staged,
 * nimbus_cop_matmul_prepared); there q_l only has to be odd and below 2^62.
 * nimbus_cop_matmul answers NIMBUS_COP_ERR_UNSUPPORTED for them.
 */
#ifndef NIMBUS_COP_H
#define NIMBUS_COP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NIMBUS_COP_OK                 0
#define NIMBUS_COP_ERR_INVALID_ARG   (-1)  /* null pointer, size or modulus out of range        */
#define NIMBUS_COP_ERR_UNSUPPORTED   (-2)  /* valid, but outside what this entry point handles  */
#define NIMBUS_COP_ERR_LAUNCH        (-3)  /* the HIP runtime refused a launch                  */
#define NIMBUS_COP_ERR_BUFFER_SIZE   (-4)  /* prepared / workspace buffer smaller than required */
#define NIMBUS_COP_ERR_STATIC_LIMIT  (-5)  /* shares exceed the built-in workspace (see below)  */

/*
 * COP accumulation + mask on the canonical layout (Algorithm 1 step 2 + step 4).
 *   X      device [m][k], entries < 2^x_bits
 *   ctW    device [k][Ch][2][L][N]
 *   moduli host   [L]
 *   mask   device [m][Ch][2][L][N], or NULL for no mask
 *   out    device [m][Ch][2][L][N]
 * Needs no setup pass and no workspace.  Where the limits of the int8 matrix-core kernel
 * allow (k <= 16383; k * Ch*2*L*N * 8 bytes and 128 * k * 8 bytes below 4 GB; not 25- to
 * 32-bit shares together with moduli above 2^55) the 64-bit words of both operands are split
 * into signed byte planes inside that kernel; everything else runs the vector-ALU kernel.
 * Same result, bit for bit, either way.
 *
 * nimbus_cop_matmul_valu always runs the vector-ALU kernel (two 32 x 32 -> 64-bit
 * multiply-adds per product, 128-bit sums, one Barrett reduction per output): any accepted
 * parameter set, and the result the matrix-core kernels are held against.
 * Additional limit of both (NIMBUS_COP_ERR_UNSUPPORTED beyond it): m <= 1,048,560.
 */
int nimbus_cop_matmul(const uint64_t *X, int m, int k, int x_bits,
                      const uint64_t *ctW, int n, int N, int L,
                      const uint64_t *moduli,
                      const uint64_t *mask, uint64_t *out, void *stream);
int nimbus_cop_matmul_valu(const uint64_t *X, int m, int k, int x_bits,
                           const uint64_t *ctW, int n, int N, int L,
                           const uint64_t *moduli,
                           const uint64_t *mask, uint64_t *out, void *stream);

/*
 * Setup phase (Section 3.2: the encrypted weights are static, sent once and
 * reused for every query).  Re-tiles the canonical ctW into the device layout
 * the matrix-core kernel streams: centred residues split into signed byte
 * planes, tile order [32-column tile][32-row k block][plane][64 lanes][16 B],
 * followed by the per-column sums of the residues.
 *   nimbus_cop_prepared_bytes  size of that buffer (0 on invalid parameters)
 *   nimbus_cop_prepare         fills it; `prepared` must be 16-byte aligned
 * Off the timed path: one call per weight matrix.
 */
size_t nimbus_cop_prepared_bytes(int k, int n, int N, int L, const uint64_t *moduli);
int nimbus_cop_prepare(const uint64_t *ctW, int k, int n, int N, int L,
                       const uint64_t *moduli,
                       void *prepared, size_t prepared_bytes, void *stream);

/*
 * COP accumulation + mask on prepared weights (same result, bit for bit, as
 * nimbus_cop_matmul on the ctW the buffer was prepared from, same k, n, N, L
 * and moduli).  Runs the int8 matrix-core kernel.  Two steps, and a call that
 * enqueues both:
 *
 *   nimbus_cop_stage_shares    X -> signed byte planes in matrix-core tile
 *                              order, written to `workspace` (the client's
 *                              shares are used as plain scalars, Section 3.2
 *                              "Row-wise Encoding"; this is only a re-layout)
 *   nimbus_cop_matmul_staged   Algorithm 1 step 2 + step 4 from staged shares
 *                              and prepared weights
 *   nimbus_cop_matmul_prepared stage_shares then matmul_staged on `stream`
 *
 *   workspace  device buffer of at least nimbus_cop_workspace_bytes(m, k,
 *              x_bits) bytes, 16-byte aligned; holds the byte planes of X.
 *              (0 is returned for invalid parameters.)
 * Additional limit (NIMBUS_COP_ERR_UNSUPPORTED beyond it): k <= 16383, so that
 * the int32 accumulators of the byte products cannot overflow.
 * Shares of more than 32 bits take two passes over the prepared weights,
 * x = x_lo + 2^32 x_hi: the pass over the upper halves leaves its reduced result
 * in `out`, the pass over the lower halves adds 2^32 times it and the mask and
 * overwrites it; the workspace holds the byte planes of both halves.
 */
size_t nimbus_cop_workspace_bytes(int m, int k, int x_bits);
int nimbus_cop_stage_shares(const uint64_t *X, int m, int k, int x_bits,
                            void *workspace, size_t workspace_bytes, void *stream);
int nimbus_cop_matmul_staged(const void *staged_shares, int m, int k, int x_bits,
                             const void *prepared, int n, int N, int L,
                             const uint64_t *moduli,
                             const uint64_t *mask, uint64_t *out, void *stream);
int nimbus_cop_matmul_prepared(const uint64_t *X, int m, int k, int x_bits,
                               const void *prepared, int n, int N, int L,
                               const uint64_t *moduli,
                               const uint64_t *mask, uint64_t *out,
                               void *workspace, size_t workspace_bytes,
                               void *stream);

/*
 * nimbus_cop_matmul_prepared for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments
 * without `workspace`, same result bit for bit.  The byte planes of X go to a buffer of
 * NIMBUS_COP_STATIC_WORKSPACE_BYTES that is part of the library's device image (each GPU
 * the library runs on holds one copy until the process ends); the call allocates and frees
 * nothing.  The device of `stream` must be the current device of the calling thread.
 *   NIMBUS_COP_ERR_STATIC_LIMIT  nimbus_cop_workspace_bytes(m, k, x_bits) exceeds the
 *                                built-in buffer (nothing is enqueued); use
 *                                nimbus_cop_matmul_prepared with a workspace of your own.
 * All calls on one GPU share that buffer: calls that may overlap in time (different
 * streams, or different threads without ordering) race on it and must use
 * nimbus_cop_matmul_prepared with separate workspaces instead.  Nothing in it has to be
 * cleared between calls: every byte a call reads it has written first.
 */
#define NIMBUS_COP_STATIC_WORKSPACE_BYTES (8u << 20)
int nimbus_cop_matmul_prepared_static(const uint64_t *X, int m, int k, int x_bits,
                                      const void *prepared, int n, int N, int L,
                                      const uint64_t *moduli,
                                      const uint64_t *mask, uint64_t *out,
                                      void *stream);

/*
 * Several calls of nimbus_cop_matmul_staged in ONE launch (Algorithm 1 steps 2 and 4 for
 * `count` independent share matrices and weight matrices of the same shape: the layers of a
 * stack whose shares are all known, the requests of a batch).  Problem i uses
 * staged_shares[i], prepared[i], masks[i] (masks = NULL, or every masks[i] = NULL: no mask;
 * otherwise a mask for every problem) and writes outs[i]; the four arrays are HOST arrays of
 * device pointers, read during the call.  Results are those of `count` separate calls, bit
 * for bit.  The kernel walks the output tiles of all problems with one workgroup per compute
 * unit and loads the first stages of a tile under the epilogue of the one before, so the
 * launch gaps and the cold start of every call but the first go away.
 * count is at most NIMBUS_COP_MAX_BATCH; shares of more than 32 bits (two passes per problem)
 * are answered NIMBUS_COP_ERR_UNSUPPORTED.  No output may overlap any buffer of the batch.
 */
#define NIMBUS_COP_MAX_BATCH 16
/* nimbus_cop_stage_shares for `count` share matrices of the same shape in one launch: X and
 * workspaces are HOST arrays of device pointers; every workspace holds workspace_bytes. */
int nimbus_cop_stage_shares_batch(int count, const uint64_t *const *X, int m, int k, int x_bits,
                                  void *const *workspaces, size_t workspace_bytes, void *stream);
int nimbus_cop_matmul_staged_batch(int count, const void *const *staged_shares, int m, int k,
                                   int x_bits, const void *const *prepared, int n, int N, int L,
                                   const uint64_t *moduli, const uint64_t *const *masks,
                                   uint64_t *const *outs, void *stream);

/*
 * Output packing (Algorithm 1 step 3; Appendix B.1 "Right Shift"; Section 3.2 "Output
 * Communication"): when n <= N/2 the payload of an output ciphertext fills only its
 * first n slots, so P = floor(N/n) of them are merged into one by negacyclic right
 * shifts, and the mask of step 4 goes onto the packed ciphertexts:
 *
 *   packed[theta] = (+)_{u in [P]} RShift(rows[theta*P + u], u*n)  (+)  mask[theta]
 *
 * RShift(ct, s) multiplies both polynomials by X^s in Z_q[X]/(X^N+1): coefficient c
 * moves to c+s, and one that passes the end re-enters at c+s-N negated.  Rows past m
 * count as zero.  (The printed algorithm garbles the shift amounts; they are the
 * multiples of the payload width n, as in the paper's figure.)
 *
 *   rows    device [m][2][L][N]: the output of a matmul entry point called with
 *           mask = NULL and the same n <= N (one ring chunk)
 *   mask    device [T][2][L][N], T = nimbus_cop_packed_count(m, n, N), residues
 *           < q_l, or NULL for no mask
 *   packed  device [T][2][L][N], canonical residues; must not alias rows
 *   nimbus_cop_packed_count  T = ceil(m / floor(N/n)); 0 for invalid arguments or n > N
 * For N/2 < n <= N there is one row per ciphertext (P = 1, T = m) and nothing to merge: a
 * caller then passes the mask to the matmul entry point, whose epilogue adds it, and does
 * not call nimbus_cop_pack at all.  (The call is still accepted; it then is a masked copy.)
 * A caller who does pack (P >= 2) passes mask = NULL to the matmul and the mask to
 * nimbus_cop_pack: Algorithm 1 masks once, after the packing.
 * Errors: NIMBUS_COP_ERR_INVALID_ARG as for the other entry points;
 * NIMBUS_COP_ERR_UNSUPPORTED for n > N (several chunks: there is nothing to pack) and
 * for more than 65535 packed ciphertexts.  On error nothing is enqueued.
 */
int nimbus_cop_packed_count(int m, int n, int N);
int nimbus_cop_pack(const uint64_t *rows, int m, int n, int N, int L,
                    const uint64_t *moduli,
                    const uint64_t *mask, uint64_t *packed, void *stream);

/*
 * Debugging aid for the value-range preconditions above, which the other entry points do
 * not test (Section 2.1: shares are elements of Z_t; Appendix B.1: ciphertext polynomials
 * have coefficients in Z_q): counts the words that break them.
 *
 *   X, ctW, mask  as for nimbus_cop_matmul (x_bits <= 64; mask may be NULL)
 *   violations    device, 3 words, written:
 *                 [0] entries of X that are >= 2^x_bits,
 *                 [1] words of ctW that are >= the modulus of their limb,
 *                 [2] words of mask that are >= the modulus of their limb (0 without mask)
 * The counts are complete when the work enqueued on `stream` has finished.
 */
int nimbus_cop_check_inputs(const uint64_t *X, int m, int k, int x_bits,
                            const uint64_t *ctW, int n, int N, int L,
                            const uint64_t *moduli,
                            const uint64_t *mask, uint64_t *violations, void *stream);

/* static, NUL-terminated description of a status code */
const char *nimbus_cop_strerror(int status);

/* library version, major*10000 + minor*100 + patch */
int nimbus_cop_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NIMBUS_COP_H */
