// Shared by the matrix-core kernels of the COP accumulation (prepared weights: cop_mfma.hip;
// canonical layout: cop_canon.hip): argument block, small helpers around the instructions the
// loops are built from, and the epilogue that turns the int32 digit sums into residues.
#pragma once
#include "cop_common.hpp"
#include <type_traits>

namespace nimbus {


typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void add128(uint64_t &hi, uint64_t &lo, uint64_t ahi, uint64_t alo)
{
    const uint64_t s = lo + alo;
    hi += ahi + (s < lo ? 1u : 0u);
    lo = s;
}

// ---------------------------------------------------------------------------
// main kernel: arguments (the pipeline is described further down)
// ---------------------------------------------------------------------------
struct MfmaArgs {
    const uint4 *xd;          // [RT][KB][DX][64] uint4
    const uint4 *planes;      // [CT][KB][DQ][64] uint4
    const uint64_t *colsum;   // [C]
    const uint64_t *mask;     // [m][C] or null
    const uint64_t *prev;     // [m][C] or null: result of the pass over the upper share halves
    uint64_t *out;            // [m][C]
    int m, KB, RB, N, L;
    uint32_t C, CT;
    uint32_t tiles;           // 128 x 64 output tiles: (CT / 2) * RB
    uint32_t kb_magic;        // floor(2^32 / KB): x / KB = umulhi(x, kb_magic) or one more
    uint32_t log_n;           // N = 2^log_n
    uint32_t l_magic;         // ceil(2^32 / L) for L >= 2: x / L = umulhi(x, l_magic) for x < 2^31
    uint32_t offx;            // OFFX
    uint64_t q[kMaxLimbs];
    double qinv[kMaxLimbs];   // 1 / q_l, rounded
    // q_l << sh
    uint64_t cst_hi[kMaxLimbs], cst_lo[kMaxLimbs];
};

// The problems of one launch: same sizes and moduli, their own shares, weights, mask and
// output.  A single call is a batch of one.
constexpr int kMaxBatch = 16;
struct ProblemPtrs {
    const uint4 *xd;            // staged shares
    const uint4 *planes;        // prepared weights
    const uint64_t *colsum;     // their column sums
    const uint64_t *mask;       // or null (all problems or none)
    uint64_t *out;
};
struct BatchPtrs {
    uint32_t count;
    uint32_t tiles_each;        // output tiles of one problem
    ProblemPtrs prob[kMaxBatch];    // (problem 0 first: one cache line with the two words above)
};

// ---- host side: constants of the argument block ----
static inline int ceil_log2(unsigned v)
{
    int b = 0;
    while ((1ull << b) < v) ++b;
    return b;
}

// OFFX: 128 in every byte of a share that can reach 128.  The same word is the XOR mask that
// turns those bytes into signed digits.
static inline uint32_t share_offset(int x_bits, int DX)
{
    uint32_t off = 0;
    for (int d = 0; d < DX; ++d)
        if (x_bits >= 8 * d + 8) off |= 0x80u << (8 * d);
    return off;
}

// q * 2^sh is added to make the signed sum non-negative: 2^sh >= k * 2^(8 DX - 1)
// bounds |sum_i x'_i c'_i| / q from above (|x'| < 2^(8 DX - 1) * 1.01, |c'| <= q / 2)
static inline int bias_shift(const Problem &p)
{
    return ceil_log2((unsigned)p.k) + 8 * planes_x(p.x_bits) - 1;
}

// everything of the argument block that follows from the problem alone: sizes, the constants
// of the tile mapping, OFFX, and per limb the modulus, its reciprocal and q << sh
// (extra_shift: one more bit of q * 2^sh for a kernel whose ciphertext digits stand for the
// residue c itself, |c'| < q, instead of the centred one, |c'| <= q / 2)
static inline void fill_common_args(const Problem &p, int DX, const uint64_t *mask,
                                    const uint64_t *prev, uint64_t *out, MfmaArgs *a,
                                    int extra_shift = 0)
{
    const int KB = kblocks(p.k);
    a->mask = mask;
    a->prev = prev;
    a->out = out;
    a->m = p.m;
    a->KB = KB;
    a->RB = (p.m + 127) / 128;
    a->N = p.N;
    a->L = p.L;
    a->C = (uint32_t)p.C;
    a->CT = (uint32_t)(p.C / kTile);
    a->tiles = (a->CT / 2u) * (uint32_t)a->RB;
    a->offx = share_offset(p.x_bits, DX);
    a->kb_magic = (uint32_t)((1ull << 32) / (uint64_t)KB);   // KB = 1: 2^32 does not fit, see below
    if (KB == 1) a->kb_magic = 0xffffffffu;
    a->log_n = 0;
    while ((1 << a->log_n) < p.N) ++a->log_n;
    a->l_magic = p.L >= 2 ? (uint32_t)(((1ull << 32) + (uint64_t)p.L - 1) / (uint64_t)p.L) : 0u;
    const int sh = bias_shift(p) + extra_shift;
    for (int l = 0; l < p.L; ++l) {
        const uint64_t q = p.limbs.limb[l].q;
        const unsigned __int128 c = (unsigned __int128)q << sh;
        a->q[l] = q;
        a->qinv[l] = 1.0 / (double)q;
        a->cst_hi[l] = (uint64_t)(c >> 64);
        a->cst_lo[l] = (uint64_t)c;
    }
}

#define NIMBUS_AS1 __attribute__((address_space(1)))
#define NIMBUS_AS3 __attribute__((address_space(3)))

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// 16 bytes per lane from LDS byte address addr + OFF
template <int OFF>
__device__ __forceinline__ v4i lds_read_b128(uint32_t addr)
{
    v4i r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
    return r;
}

// wait until at most PENDING of this wave's LDS reads are outstanding; tied to the
// register that the oldest still-awaited read fills so that its users stay behind it
template <int PENDING>
__device__ __forceinline__ void wait_lds(v4i &x)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(PENDING) : "memory");
}

// keeps the users of x behind the preceding volatile asm statements (and the producer of
// x before the following ones)
__device__ __forceinline__ void tie(v4i &x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void tie_acc(v16i &x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void tie(int &x) { asm volatile("" : "+v"(x)); }

// wait until at most PENDING of this wave's global loads (here: direct-to-LDS loads) are
// outstanding
template <int PENDING>
__device__ __forceinline__ void wait_vmem()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PENDING) : "memory");
}

// one wave copies 64 x 16 B (a whole operand tile) from global memory straight into LDS;
// lane l's bytes land at dst + l*16.  The source is a buffer descriptor (wave-uniform base)
// plus a per-lane offset plus a wave-uniform offset: the address needs no vector arithmetic.
// STREAM puts the streaming hint on the load.  With one row block per column tile every
// ciphertext byte is read once and should not push the X planes out of L2 (for the X
// planes, which all workgroups of an XCD read within a few microseconds of each other, the
// hint makes no measurable difference, and one kind of load lets all eight waves run the
// same instructions).  With several row blocks per column tile the hint is left off: the
// tile has to stay in the XCD's L2 until the last of them has read it.
template <bool STREAM>
__device__ __forceinline__ void dma_tile(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_off,
                                         uint32_t uniform_off, void *dst_wave)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (NIMBUS_AS3 void *)dst_wave, 16, lane_off,
                                             uniform_off, 0, STREAM ? 2 : 0);
}

// Wait until at most n of this wave's loads are pending, 0 <= n <= 63, n wave-uniform.
// The count is an immediate of the wait instruction: jump into a table of 64 entries
// of 8 bytes, entry i = { wait for at most i pending; branch to the end }.  The distance
// from the program counter that was read to the table is left to the assembler.
__device__ __forceinline__ void wait_vmem_n(int n)
{
    asm volatile(
        "s_getpc_b64 s[96:97]\n"
        ".Lwait_vmem_pc_%=:\n\t"
        "s_lshl_b32 s98, %0, 3\n\t"
        "s_add_u32 s98, s98, .Lwait_vmem_table_%=-.Lwait_vmem_pc_%=\n\t"
        "s_add_u32 s96, s96, s98\n\t"
        "s_addc_u32 s97, s97, 0\n\t"
        "s_setpc_b64 s[96:97]\n"
        ".Lwait_vmem_table_%=:\n\t"
        ".irp cnt,0,1,2,3,4,5,6,7,8,9,10,11,12,13,14,15,16,17,18,19,20,21,22,23,24,25,26,27,28,29,30,31,"
        "32,33,34,35,36,37,38,39,40,41,42,43,44,45,46,47,48,49,50,51,52,53,54,55,56,57,58,59,60,61,62,63\n\t"
        "s_waitcnt vmcnt(\\cnt)\n\t"
        "s_branch .Lwait_vmem_end_%=\n\t"
        ".endr\n"
        ".Lwait_vmem_end_%=:"
        :
        : "s"(__builtin_amdgcn_readfirstlane(n))
        : "s96", "s97", "s98", "scc", "memory");
}

// Wait until at most W * n of this wave's loads are pending, for n in [NLO, NHI] with
// NHI - NLO <= 2, n wave-uniform: a short chain of compares in the order the code runs
// through, instead of the table jump above.
template <int W, int NHI, int NLO>
__device__ __forceinline__ void wait_vmem_loads(int n)
{
    static_assert(NHI - NLO <= 2 && NHI >= NLO, "at most three cases");
    if constexpr (NHI == NLO) {
        wait_vmem<W * NHI>();
    } else if constexpr (NHI - NLO == 1) {
        asm volatile("s_cmp_eq_u32 %0, %1\n\t"
                     "s_cbranch_scc1 .Lwl_hi_%=\n\t"
                     "s_waitcnt vmcnt(%2)\n\t"
                     "s_branch .Lwl_end_%=\n"
                     ".Lwl_hi_%=:\n\t"
                     "s_waitcnt vmcnt(%3)\n"
                     ".Lwl_end_%=:"
                     :
                     : "s"(n), "n"(NHI), "n"(W * NLO), "n"(W * NHI)
                     : "scc", "memory");
    } else {
        asm volatile("s_cmp_eq_u32 %0, %1\n\t"
                     "s_cbranch_scc1 .Lwl_hi_%=\n\t"
                     "s_cmp_eq_u32 %0, %2\n\t"
                     "s_cbranch_scc1 .Lwl_mid_%=\n\t"
                     "s_waitcnt vmcnt(%3)\n\t"
                     "s_branch .Lwl_end_%=\n"
                     ".Lwl_mid_%=:\n\t"
                     "s_waitcnt vmcnt(%4)\n\t"
                     "s_branch .Lwl_end_%=\n"
                     ".Lwl_hi_%=:\n\t"
                     "s_waitcnt vmcnt(%5)\n"
                     ".Lwl_end_%=:"
                     :
                     : "s"(n), "n"(NHI), "n"(NHI - 1), "n"(W * NLO), "n"(W * (NHI - 1)), "n"(W * NHI)
                     : "scc", "memory");
    }
}

// ---------------------------------------------------------------------------
// epilogue: rebuild the sums from the diagonals, add the constant and the mask, reduce, store
//   mask, prev, out  the problem's mask (or null), the result of the pass over the upper share
//              halves (or null) and its output, [m][C] each
//   acc        the wave's ND = DX + DQ - 1 accumulator tiles (32 x 32 outputs: element r of
//              the lane is row row0 + 8 (r / 4) + r % 4, column col)
//   limb       limb of the wave's 32 columns;  colsum_S  sum of the column's residues mod q
//   row0, col  the lane's first row and its column in the whole output
//   mask_tile  MASKLDS: the lane's word of row0 in the workgroup's mask tile in LDS
// ---------------------------------------------------------------------------
template <int ND, bool FULL, bool MASKLDS>
__device__ __forceinline__ void cop_epilogue(v16i (&acc)[ND], const MfmaArgs &a,
                                             const uint64_t *mask, const uint64_t *prev,
                                             uint64_t *out, uint32_t limb, uint64_t colsum_S,
                                             int row0, uint32_t col, const unsigned char *mask_tile)
{
    const uint64_t q = a.q[limb];
    const double qinv = a.qinv[limb];
    // every load of the epilogue first (mask words, then the column sum), so that their
    // latencies overlap
    // element r of the lane is row row0 + roff(r); addresses are the lane's address of
    // row0 plus a wave-uniform multiple of the row length
    auto roff = [](int r) -> int { return 8 * (r >> 2) + (r & 3); };
    const size_t lane_elem = (size_t)row0 * a.C + col;
    const uint64_t *const mask0 = mask ? mask + lane_elem : nullptr;
    const uint64_t *const prev0 = prev ? prev + lane_elem : nullptr;
    uint64_t *const out0 = out + lane_elem;
    uint64_t mk[16];                                // read once: streaming loads
    if constexpr (MASKLDS) {
        // the tile is in LDS, row-major [128][64] words; mask_tile is the lane's word of row0
#pragma unroll
        for (int r = 0; r < 16; ++r) mk[r] = *(const uint64_t *)(mask_tile + roff(r) * 512);
    } else if (mask) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            mk[r] = (FULL || row0 + roff(r) < a.m)
                        ? __builtin_nontemporal_load(&mask0[(size_t)roff(r) * a.C])
                        : 0;
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) mk[r] = 0;
    }
    uint64_t cst_hi = a.cst_hi[limb], cst_lo = a.cst_lo[limb];
    {
        const uint64_t S = colsum_S;
        add128(cst_hi, cst_lo, __umul64hi(S, (uint64_t)a.offx), S * (uint64_t)a.offx);
    }
    // V = cst + mask + sum_d D_d 256^d, 0 <= V < 2^47 q.  Two things are needed of V: its
    // low 64 bits, exactly, and V / q to within 1/2.  The diagonals are first gathered four
    // at a time into exact 64-bit integers with signed 32 x 32 + 64-bit multiply-adds,
    //     g0 = c0 + sum_{d<4} D_d 256^d,   g1 = c1 + sum_{4<=d<8} D_d 256^(d-4),
    // (c0, c1: the two low 32-bit words of cst; |g| < 2^56), so that
    //     V = (g0 + mask) + 2^32 g1 + 2^64 (cst_hi + sum_{d>=8} D_d 256^(d-8)).
    // Low bits: those of g0 + mask, with the low word of g1 added to the upper word.
    // Quotient: the three terms in double precision.  The third is exact (below 2^53);
    // g1 and g0 + mask each round once when they are converted; every partial sum is a
    // prefix of the signed-digit expansion and stays below 4 * 2^sh q in magnitude (the
    // digit magnitudes of an operand add up to at most twice its bound), so the handful of
    // roundings (eight at most, each below 2^-53 * 2^47 = 2^-6 of a quotient unit) leave the
    // estimate off by well under 1/4.  With 1/2 taken off, rounded to a multiple of 1/4 and
    // then down, it is floor(V/q) or one less, never more; the remainder is then formed
    // modulo 2^64 and corrected once.
    const double two32 = 4294967296.0;
    const int64_t c0 = (int64_t)(cst_lo & 0xffffffffu), c1 = (int64_t)(cst_lo >> 32);
    // cst < 2^108 (q << sh < 2^107, OFFX * S < 2^94): its upper word converts exactly
    const double k2 = fma((double)(uint32_t)(cst_hi >> 32), two32, (double)(uint32_t)cst_hi) *
                      (two32 * two32);
    // (wave-uniform: the limb follows from the wave's column tile)
    const uint32_t q_lo = __builtin_amdgcn_readfirstlane((uint32_t)q);
    const uint32_t q_hi = __builtin_amdgcn_readfirstlane((uint32_t)(q >> 32));
    const uint32_t nq_lo = __builtin_amdgcn_readfirstlane((uint32_t)(0 - q));           // 2^64 - q
    const uint32_t nq_hi = __builtin_amdgcn_readfirstlane((uint32_t)((0 - q) >> 32));
    // First everything that does not need the mask words (their loads are in flight), then,
    // per element, mask, quotient, remainder, store.
    // (the powers of 256 are kept opaque so that each term is one multiply-add instead of a
    // sign extension, a 64-bit shift and a 64-bit add)
    int32_t pow256[4] = {1, 1 << 8, 1 << 16, 1 << 24};
#pragma unroll
    for (int d = 0; d < 4; ++d) asm volatile("" : "+s"(pow256[d]));
    static_assert(ND >= 8, "two full groups of diagonals");
    int64_t g0[16];
    uint32_t g1_lo[16];
    double v_hi[16];                                // 2^32 g1 + 2^64 (...), in double
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        auto D = [&](int d) -> int32_t { return acc[d][r]; };
        int64_t s0 = c0, s1 = c1;
#pragma unroll
        for (int d = 0; d < 4; ++d) s0 += (int64_t)D(d) * (int64_t)pow256[d];
#pragma unroll
        for (int d = 4; d < 8; ++d) s1 += (int64_t)D(d) * (int64_t)pow256[d - 4];
        double top = k2, scale = two32 * two32;
#pragma unroll
        for (int d = 8; d < ND; ++d) {
            top = fma((double)D(d), scale, top);
            scale *= 256.0;
        }
        g0[r] = s0;
        g1_lo[r] = (uint32_t)s1;
        const double s1_d = fma((double)(int32_t)(s1 >> 32), two32, (double)(uint32_t)s1);
        v_hi[r] = fma(s1_d, two32, top);
    }
    // the second half stays behind the first: volatile statements keep their order, and
    // these make the first half's results and the loaded words pass through them
#pragma unroll
    for (int r = 0; r < 16; ++r) asm volatile("" : "+v"(g0[r]), "+v"(g1_lo[r]), "+v"(v_hi[r]));
    // Shares wider than 32 bits take two passes, x = x_lo + 2^32 x_hi: the second one adds
    // 2^32 times the (reduced) result of the pass over the upper halves, read from where
    // this pass writes its own result (prev may be out: an element is read and written by
    // the same lane, and every read comes before the first write).  2^32 prev < 2^32 q keeps
    // V below 2^47 q.  (A block of its own behind one wave-uniform branch: the narrow path
    // does not execute any of it.)
    if (prev) {
        uint64_t pv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r)
            pv[r] = (FULL || row0 + roff(r) < a.m) ? __builtin_nontemporal_load(&prev0[(size_t)roff(r) * a.C]) : 0;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            g1_lo[r] += (uint32_t)pv[r];
            // exact below 2^53; above, off by < 2^-53 of a term that is < 2^32 q
            v_hi[r] = fma(fma((double)(uint32_t)(pv[r] >> 32), two32, (double)(uint32_t)pv[r]),
                          two32, v_hi[r]);
        }
        asm volatile("" ::: "memory");
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) asm volatile("" : "+v"(mk[r]));
    // wave-uniform constants of the quotient estimate, kept in vector registers
    // (the constant starts out in scalar registers behind an opaque statement: a caller that
    // runs this epilogue in a loop would otherwise have it built once in front of the loop
    // and carried, or spilled, through all of it)
    uint64_t magic_bits = 0x4317fffffffffffeull;                   // 3 * 2^49 - 1/2 as a double
    asm volatile("" : "+s"(magic_bits));
    double qinv_v = qinv, magic_c = __builtin_bit_cast(double, magic_bits);
    // (the subtract-with-borrow reads vcc, which leaves no room for a second scalar operand)
    uint32_t q_hi_v = q_hi;
    asm volatile("" : "+v"(qinv_v), "+v"(magic_c), "+v"(q_hi_v));
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int64_t t0 = g0[r] + (int64_t)mk[r];          // |g0| < 2^56, mask < 2^62
        const uint32_t lo_lo = (uint32_t)t0;
        const uint32_t lo_hi = (uint32_t)(t0 >> 32) + g1_lo[r];
        // quotient estimate
        const double vd = v_hi[r] + fma((double)(int32_t)(t0 >> 32), two32, (double)lo_lo);
        // est = V/q - 1/2 rounded to a multiple of 1/4, then down to an integer: the constant
        // 3 * 2^49 - 1/2 puts the sum into [2^50, 2^51), where doubles are 1/4 apart, so bits
        // 2..51 of the sum hold est + 2^49 (est > -2^48).  With the estimate of V/q off by
        // less than 1/4, est is floor(V/q) or one less (-1 is possible for V < q); only est
        // modulo 2^64 is needed, and the signed field extract gives its upper word.
        // (written out as one instruction: the compiler would rebuild the constant in a
        // fresh register pair for every element to feed a two-operand multiply-add)
        double magic;
        asm("v_fma_f64 %0, %1, %2, %3" : "=v"(magic) : "v"(vd), "v"(qinv_v), "v"(magic_c));
        const uint64_t mbits = __builtin_bit_cast(uint64_t, magic);
        const uint32_t m_hi = (uint32_t)(mbits >> 32);
        const uint32_t ql = (uint32_t)(mbits >> 2);
        const uint32_t qh = (uint32_t)__builtin_amdgcn_sbfe((int32_t)m_hi, 2, 17);
        // remainder modulo 2^64: lo - (qh 2^32 + ql) q = lo + (qh 2^32 + ql) (2^64 - q), in
        // [0, 2q); then one correction.  (With the negated modulus the lower product goes into
        // one multiply-add on top of lo, and nothing has to be subtracted with borrow.)
        const uint64_t t = (uint64_t)ql * nq_lo + (((uint64_t)lo_hi << 32) | lo_lo);
        const uint32_t t_lo = (uint32_t)t;
        const uint32_t t_hi = (uint32_t)(t >> 32) + (ql * nq_hi + qh * nq_lo);   // upper word only
        // res = t - q if that does not borrow, else t (subtract with borrow, then select on
        // the borrow; a value written to vcc may be read two wait states later)
        uint32_t r_lo, r_hi;
        asm("v_subrev_co_u32_e32 %0, vcc, %4, %2\n\t"
            "s_nop 1\n\t"
            "v_subbrev_co_u32_e32 %1, vcc, %5, %3, vcc\n\t"
            "s_nop 1\n\t"
            "v_cndmask_b32_e32 %0, %0, %2, vcc\n\t"
            "v_cndmask_b32_e32 %1, %1, %3, vcc"
            : "=&v"(r_lo), "=&v"(r_hi)
            : "v"(t_lo), "v"(t_hi), "s"(q_lo), "v"(q_hi_v)
            : "vcc");
        const uint64_t res = ((uint64_t)r_hi << 32) | r_lo;
        // (streaming store: the output is not read again by this kernel, and lines that do
        // not sit dirty in L2 need no write-back when the kernel ends)
        if (FULL || row0 + roff(r) < a.m) __builtin_nontemporal_store(res, &out0[(size_t)roff(r) * a.C]);
    }
}

}  // namespace nimbus
