// Transform kernels of the server side (see rlwe.hip for the method): the arithmetic, the
// rounds, the kernel that multiplies a polynomial by the secret, and the launches that pick
// its instance.  Shared by the translation units that instantiate the kernel for the phase
// (rlwe.hip) and for the encryption (rlwe_encrypt.hip): the instances of one unit take minutes
// to compile, side by side they take half as long.
#pragma once

#include "cop_common.hpp"
#include "../../include/nimbus_cop.h"
#include "../../include/nimbus_rlwe.h"

namespace nimbus {

typedef unsigned __int128 u128;

constexpr int kRlweMinLogN = 5;
constexpr int kRlweMaxLogN = 15;        // 2^14 coefficients (128 KiB of the 160 KiB LDS) at a time

struct Twiddle {
    uint64_t w;     // < q
    uint64_t ws;    // floor(w * 2^64 / q)
};

// Per limb three sets of  forward powers | inverse powers | transformed secret (times 1/N),
// N entries each: set 0 in the natural order (bit-reversed powers, secret by coefficient), sets
// 1 and 2 the same entries in the order in which the product kernels for large and for small
// batches read them (see table_slot()).
constexpr int kTableSets = 3;
__host__ __device__ inline size_t set_entries(int N) { return (size_t)3 * (size_t)N; }
__host__ __device__ inline size_t limb_table_entries(int N) { return kTableSets * set_entries(N); }

struct RlweLimb {
    Limb red;           // constants of the one-shot reduction of a 128-bit value
    uint64_t psi;       // primitive 2N-th root of unity mod q (setup only)
    uint64_t psi_inv;   // its inverse (setup only)
    uint64_t n_inv;     // N^-1 mod q (setup only)
    uint64_t delta;     // floor(Q / t) mod q (encryption only)
    uint32_t fold_m;    // floor(2^(64 + fold_k) / q), below 2^32 (see fold(); q >= 2^34 only)
    uint32_t fold_k;    // bit length of q minus 33
};

struct RlweArgs {
    RlweLimb limb[kMaxLimbs];
};

// With nq = 2^64 - q the same value is  x w + floor(x w' / 2^64) nq  (mod 2^64): the multiply-add
// chain of the second product takes the first as its addend, and no borrow travels through a
// scalar register.  nq comes from negated(), which keeps the compiler from turning the sum
// back into a difference.
__device__ __forceinline__ uint64_t negated(uint64_t q)
{
    uint64_t nq = 0 - q;
    asm volatile("" : "+s"(nq));
    return nq;
}
__device__ __forceinline__ uint64_t mul_lazy(uint64_t x, const Twiddle &t, uint64_t nq)
{
    return x * t.w + __umul64hi(x, t.ws) * nq;
}

// The same product with a quotient estimate from three of the four partial products,
//   h = x1 w1' + floor(x0 w1' / 2^32) + floor(x1 w0' / 2^32)   (x = x1 2^32 + x0, w' = w1' 2^32 + w0'),
// which falls short of floor(x w' / 2^64) by at most 2: the result lies in [0, 4q).  Five
// instructions fewer; for moduli that leave the room (see group_butterflies).
__device__ __forceinline__ uint64_t mul_loose(uint64_t x, const Twiddle &t, uint64_t nq)
{
    const uint32_t x0 = (uint32_t)x, x1 = (uint32_t)(x >> 32);
    const uint32_t w0 = (uint32_t)t.ws, w1 = (uint32_t)(t.ws >> 32);
    const uint64_t h = (uint64_t)x1 * w1 + __umulhi(x0, w1) + __umulhi(x1, w0);
    return x * t.w + h * nq;
}

// u >= m ? u - m : u  for  m <= 2^63 and u < m + 2^63, given nm = negated(m): decided by the
// sign of the sum, one 64-bit add and a test of the upper word
__device__ __forceinline__ uint64_t cond_sub(uint64_t u, uint64_t nm)
{
    const uint64_t d = u + nm;
    return (int32_t)(d >> 32) < 0 ? u : d;
}

// One modulus as the butterflies use it.
struct Mod {
    uint64_t q, two_q;
    uint64_t nq, n2q;           // 2^64 - q, 2^64 - 2q
    uint32_t fold_m, fold_k;
};
__device__ __forceinline__ Mod make_mod(const RlweLimb &P)
{
    return Mod{P.red.q, 2 * P.red.q, negated(P.red.q), negated(2 * P.red.q), P.fold_m, P.fold_k};
}

// Any 64-bit x -> a value below 2q congruent to it, for 2^34 <= q: the quotient estimate
//   h = floor(floor(x / 2^32) m / 2^(32+k)),  m = floor(2^(64+k) / q),  k = bitlen(q) - 33 >= 1,
// falls short of x / q by less than  x / 2^(64+k) + 2^32 / q + 1 <= 2, and never exceeds it.
__device__ __forceinline__ uint64_t fold(uint64_t x, const Mod &md)
{
    const uint32_t h = __umulhi((uint32_t)(x >> 32), md.fold_m) >> md.fold_k;
    return x + (uint64_t)h * md.nq;
}

// a, b < q  ->  a b mod q
__device__ __forceinline__ uint64_t mulmod(uint64_t a, uint64_t b, const Limb &P)
{
    return barrett128(__umul64hi(a, b), a * b, P);
}

// ---------------------------------------------------------------------------
// the transform rounds
// ---------------------------------------------------------------------------
// MAXS: most stages a round may take (2^MAXS coefficients per thread and round).  Large
// batches use 4: fewest trips through the LDS.  A batch that cannot fill the chip takes
// fewer stages per round and more threads per polynomial instead: shorter dependent chains
// per thread, more waves to hide the latencies of one polynomial.
constexpr int rounds_for(int stages, int MAXS) { return (stages + MAXS - 1) / MAXS; }
// stages of the next round when `stages` are left: as even a split as possible
constexpr int round_stages(int stages, int MAXS)
{
    return (stages + rounds_for(stages, MAXS) - 1) / rounds_for(stages, MAXS);
}
constexpr int threads_for(int logN, int MAXS)
{
    const int t = (1 << logN) >> MAXS;
    return t < 64 ? 64 : (t > 1024 ? 1024 : t);
}
// Order of the table entries a product kernel reads.  A thread of a round over the stages
// P0 .. P0+S-1 handles block i0 of stage P0 and needs, of stage P0+st, the 2^st entries
// (i0 << st) + j: in the natural order the threads of a wave read with a stride of 2^st entries,
// and the late stages cost a cache line per lane.  The kernels' sets hold the entries of such a
// stage as  (j << P0) + i0  instead: the lanes of a wave read neighbours.  Likewise the
// transformed secret of the round in the middle, coefficient (g << S) + r of group g, sits
// at (r << (logN - S)) + g.  The stages below `pre` (done outside the rounds) keep their place.
__host__ __device__ inline int power_slot(int logN, int pre, int maxs, int e)
{
    if (e < (1 << pre) || e < 1) return e;
    int s = 0;
    while ((2 << s) <= e) ++s;                      // stage of entry e: 2^s <= e < 2^(s+1)
    int p0 = pre;
    while (p0 + round_stages(logN - p0, maxs) <= s) p0 += round_stages(logN - p0, maxs);
    const int st = s - p0, b = e - (1 << s);
    const int i0 = b >> st, j = b & ((1 << st) - 1);
    return (1 << s) + (j << p0) + i0;
}
__host__ __device__ inline int secret_slot(int logN, int pre, int maxs, int c)
{
    int p0 = pre;
    while (p0 + round_stages(logN - p0, maxs) < logN) p0 += round_stages(logN - p0, maxs);
    const int S = logN - p0;                        // stages of the round in the middle
    return ((c & ((1 << S) - 1)) << (logN - S)) + (c >> S);
}

// LDS index of coefficient i: one word of padding after every 16, so that the strides of
// 16 and 256 words of the later rounds spread over the banks
__device__ __forceinline__ int pad(int i) { return i + (i >> 4); }
constexpr int padded_size(int N) { return N + (N >> 4); }

enum RoundKind { kForward, kInverse, kMiddle };

// One round over the stages P0 .. P0+S-1.  A group is the 2^S coefficients
//   base + r * 2^LT,  r < 2^S,  base = i0 * 2^(LOGN-P0) + o,  o < 2^LT,  LT = LOGN - P0 - S:
// block i0 of stage P0 (2^P0 blocks), offset o inside the smallest stride of the round.
// In stage P0+st coefficient r of the group sits in block i0 * 2^st + (r >> (S - st)), so the
// stage uses 2^st table entries per group, 2^S - 1 per direction in all.
template <int LOGN, int P0, int S>
struct Group {
    static constexpr int N = 1 << LOGN, R = 1 << S, LT = LOGN - P0 - S, G = N / R;
    int i0, base;
    // (a round from stage 0 has one block: written out, so that its table indices are constants)
    __device__ __forceinline__ explicit Group(int g)
        : i0(P0 == 0 ? 0 : g >> LT),
          base(P0 == 0 ? g : ((g >> LT) << (LOGN - P0)) + (g & ((1 << LT) - 1))) {}
    __device__ __forceinline__ int at(int r) const { return base + (r << LT); }
    // pad(at(r) - index0) = pad(base - index0) + a constant: r << LT has no bits below LT, the
    // rest of the index none between LT and LT + S, and index0 and the block's start are
    // multiples of 2^(LT+S); needs LT >= 4 or LT + S >= 4
    static constexpr bool kSeparable = LT + S >= 4;
    static constexpr int padded_step(int r) { return (r << LT) + ((r << LT) >> 4); }
    // table index of entry j (j < 2^st) of stage st: in the natural order, and in a kernel's set
    // (power_slot())
    template <bool OWN_SET>
    __device__ __forceinline__ int entry(int st, int j) const
    {
        return OWN_SET ? (1 << (P0 + st)) + (j << P0) + i0 : (1 << (P0 + st)) + (i0 << st) + j;
    }
    // index of the transformed secret for coefficient r of group g (round in the middle: LT = 0)
    template <bool OWN_SET>
    __device__ __forceinline__ int secret(int r, int g) const
    {
        return OWN_SET ? (r << (LOGN - S)) + g : at(r);
    }
};

// The table entries one group needs in one round, in registers: loaded before the barrier
// that ends the round before, so that their latency does not come after it.
template <int S, RoundKind KIND>
struct RoundTable {
    static constexpr int R = 1 << S;
    static constexpr int NF = KIND != kInverse ? R - 1 : 1;
    static constexpr int NI = KIND != kForward ? R - 1 : 1;
    static constexpr int NS = KIND == kMiddle ? R : 1;
    Twiddle f[NF], i[NI], s[NS];
};

template <int LOGN, int P0, int S, RoundKind KIND>
__device__ __forceinline__ RoundTable<S, KIND> load_round_table(const Twiddle *__restrict__ fwd,
                                                                const Twiddle *__restrict__ inv,
                                                                const Twiddle *__restrict__ shat,
                                                                int g)
{
    // (only the product kernels ask ahead: the tables are their own set)
    const Group<LOGN, P0, S> grp(g);
    RoundTable<S, KIND> t;
#pragma unroll
    for (int st = 0; st < S; ++st)
#pragma unroll
        for (int j = 0; j < (1 << st); ++j) {
            if constexpr (KIND != kInverse) t.f[(1 << st) - 1 + j] = fwd[grp.template entry<true>(st, j)];
            if constexpr (KIND != kForward) t.i[(1 << st) - 1 + j] = inv[grp.template entry<true>(st, j)];
        }
    if constexpr (KIND == kMiddle) {
#pragma unroll
        for (int r = 0; r < (1 << S); ++r) t.s[r] = shat[grp.template secret<true>(r, g)];
    }
    return t;
}

// Two ways of keeping the values inside 64 bits.
//
// Any modulus below 2^62 (LAZY = kNever): forward values stay below 4q (one conditional
// subtraction of 2q per butterfly), inverse values below 2q (one per sum).
//
// Moduli from 2^34 to 2^58 (LAZY = kLoose) leave room for 64 multiples of q in a word.
// Then the products take the cheaper quotient estimate of mul_loose() (below 4q instead of 2q)
// and the conditional subtractions go:
//   forward: a value that enters a stage below B q leaves it below (B + 4) q; inputs below 3q
//            (q, or 3q behind the stage done on the way in) and at most 14 more stages, or q
//            and 15 stages: below 61q;
//   inverse: the bound of every register is known when the code is compiled: a product is
//            below 4q, a sum below the sum of its operands' bounds, u - v is made non-negative
//            by adding (bound of v) q; the first register of a group of 2^S doubles S times.
//            At the end of a round the registers whose bound exceeds `tout` are folded below 2q
//            (five instructions each, fold()); tout is 64 / 2^(stages of the next round), so
//            that the next round cannot overflow, and 2 in the last round, whose results are
//            all below 2q.
// Moduli from 2^58 to 2^59 (LAZY = kTight; the 59-bit limb of the paper's 64-bit setting): room
// for 32 multiples; the same scheme with the exact product (below 2q): forward below 31q, and
// tout = 32 / 2^(stages of the next round).
enum Lazy { kNever = 0, kLoose = 1, kTight = 2 };
constexpr unsigned lazy_units(int lazy) { return lazy == kLoose ? 64 : 32; }
constexpr unsigned product_units(int lazy) { return lazy == kLoose ? 4 : 2; }   // mul_loose() / mul_lazy()
constexpr unsigned kFoldUnits = 2;      // bound of fold()

// bound (in multiples of q) of the largest register of a group after an inverse round of S
// stages that starts from `bin` everywhere and folds what exceeds `tout`
constexpr unsigned inverse_round_out(int S, unsigned bin, unsigned tout, unsigned prod)
{
    unsigned b[16] = {};
    const int R = 1 << S;
    for (int r = 0; r < R; ++r) b[r] = bin;
    for (int st = S - 1; st >= 0; --st) {
        const int half = R >> (st + 1);
        for (int r = 0; r < R; ++r) {
            if (r & half) continue;
            b[r] += b[r + half];
            b[r + half] = prod;
        }
    }
    unsigned most = 0;
    for (int r = 0; r < R; ++r) {
        const unsigned v = b[r] > tout ? kFoldUnits : b[r];
        most = v > most ? v : most;
    }
    return most;
}

// the butterflies of one group; F(st, j), I(st, j), Sh(r) hand out the table entries.
// BIN, TOUT: with LAZY, bound of the registers at the start of the inverse stages, and the
// bound above which a register is folded after them (both in multiples of q).
template <int S, RoundKind KIND, int LAZY, unsigned BIN, unsigned TOUT, typename FwdT, typename InvT,
          typename SecT>
__device__ __forceinline__ void group_butterflies(uint64_t (&x)[1 << S], const Mod &md, FwdT F, InvT I,
                                                  SecT Sh)
{
    constexpr int R = 1 << S;
    static_assert(S <= 4, "bounds are tracked for up to 16 registers");
    constexpr unsigned PROD = product_units(LAZY);
    auto product = [&](uint64_t v, const Twiddle &t) {
        return LAZY == kLoose ? mul_loose(v, t, md.nq) : mul_lazy(v, t, md.nq);
    };
    if constexpr (KIND != kInverse) {
#pragma unroll
        for (int st = 0; st < S; ++st) {
            const int half = R >> (st + 1);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (r & half) continue;
                const Twiddle t = F(st, r >> (S - st));
                const uint64_t u = LAZY != kNever ? x[r] : cond_sub(x[r], md.n2q);
                const uint64_t v = product(x[r + half], t);
                x[r] = u + v;
                x[r + half] = u + PROD * md.q - v;
            }
        }
    }
    if constexpr (KIND == kMiddle) {
        // Sh(r): the transformed secret at the group's coefficient r (bit-reversed position = index
        // in the LDS; where in the table that is, the caller knows)
#pragma unroll
        for (int r = 0; r < R; ++r)
            x[r] = product(x[r], Sh(r));
    }
    if constexpr (KIND != kForward) {
        if constexpr (LAZY != kNever) {
            static_assert(((KIND == kMiddle ? PROD : BIN) << S) <= lazy_units(LAZY), "inverse round overflows");
            unsigned b[R];          // folded away: every index below is a constant after unrolling
#pragma unroll
            for (int r = 0; r < R; ++r) b[r] = KIND == kMiddle ? PROD : BIN;
#pragma unroll
            for (int st = S - 1; st >= 0; --st) {
                const int half = R >> (st + 1);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (r & half) continue;
                    const Twiddle t = I(st, r >> (S - st));
                    const uint64_t u = x[r], v = x[r + half];
                    x[r] = u + v;
                    x[r + half] = product(u + b[r + half] * md.q - v, t);
                    b[r] += b[r + half];
                    b[r + half] = PROD;
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (b[r] > TOUT) x[r] = fold(x[r], md);
        } else {
#pragma unroll
            for (int st = S - 1; st >= 0; --st) {
                const int half = R >> (st + 1);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (r & half) continue;
                    const Twiddle t = I(st, r >> (S - st));
                    const uint64_t u = x[r], v = x[r + half];
                    x[r] = cond_sub(u + v, md.n2q);
                    x[r + half] = mul_lazy(u + md.two_q - v, t, md.nq);
                }
            }
        }
    }
}

// A ring too large for the LDS (2^15 coefficients) is handled in 2^PRE parts: the stages
// below PRE are done on the way in (forward) and in a pass of their own afterwards
// (inverse), and between them every part is a transform of 2^(LOGN-PRE) coefficients with
// its own table entries.  Part h holds the coefficients h * 2^(LOGN-PRE) ... of the ring
// (blocks of the stages from PRE on never straddle two parts), so its groups are the ring's
// groups  h * G / 2^PRE ... and its LDS index is the ring index minus h * 2^(LOGN-PRE).
struct Part {
    int group0;     // first group of the part (in the numbering of the round at hand)
    int index0;     // first coefficient of the part
};
template <int LOGN, int PRE, int S>
__device__ __forceinline__ Part part_of(int h)
{
    return Part{h * (((1 << LOGN) >> S) >> PRE), h << (LOGN - PRE)};
}

// Where a round's coefficients come from and go to.  The first and the last round of a product
// (stages from 0, one group per thread) use the very coefficients a thread loads from and
// stores to memory in coalesced order (group g: g + r * threads), so they can take them from
// and leave them in registers `xio` instead of the LDS.
enum RoundIo { kLdsToLds, kRegsToLds, kLdsToRegs };

// a round with the table entries read from memory inside it (any number of groups per thread)
// OWN_SET: the tables are the kernel's own set (see power_slot()), else the natural order.
template <int LOGN, int PRE, int P0, int S, RoundKind KIND, int NT, int LAZY = kNever, unsigned BIN = 2,
          unsigned TOUT = 2, RoundIo IO = kLdsToLds, bool OWN_SET = false>
__device__ __forceinline__ void ntt_round(uint64_t *lds, const Twiddle *__restrict__ fwd,
                                          const Twiddle *__restrict__ inv,
                                          const Twiddle *__restrict__ shat, const Mod &md, int tid,
                                          int h, uint64_t *xio = nullptr)
{
    using Grp = Group<LOGN, P0, S>;
    static_assert(IO == kLdsToLds || (PRE == 0 && P0 == 0 && Grp::G == NT), "one group per thread");
    const Part part = part_of<LOGN, PRE, S>(h);
    // In a round from stage 0 every thread needs the same table entries: read through the
    // scalar cache.  Apart from the registers this keeps them out of the queue of the vector
    // loads, which completes in order: the loads from HBM that the caller has issued in front of
    // its last round (what is added to the product) then hold up nothing in that round.
    auto entry_of = [](const Twiddle *table, int index) -> Twiddle {
        if constexpr (PRE == 0 && P0 == 0) {
            typedef const __attribute__((address_space(4))) Twiddle *Uniform;
            const Uniform at = (Uniform)table + index;
            return Twiddle{at->w, at->ws};
        } else {
            return table[index];
        }
    };
    for (int g = tid; g < (Grp::G >> PRE); g += NT) {
        const Grp grp(part.group0 + g);
        uint64_t x[Grp::R];
        const int p0 = pad(grp.base - part.index0);
        auto slot = [&](int r) {
            return Grp::kSeparable ? p0 + Grp::padded_step(r) : pad(grp.at(r) - part.index0);
        };
#pragma unroll
        for (int r = 0; r < Grp::R; ++r) x[r] = IO == kRegsToLds ? xio[r] : lds[slot(r)];
        group_butterflies<S, KIND, LAZY, BIN, TOUT>(
            x, md, [&](int st, int j) { return entry_of(fwd, grp.template entry<OWN_SET>(st, j)); },
            [&](int st, int j) { return entry_of(inv, grp.template entry<OWN_SET>(st, j)); },
            [&](int r) { return shat[grp.template secret<OWN_SET>(r, part.group0 + g)]; });
#pragma unroll
        for (int r = 0; r < Grp::R; ++r) {
            if constexpr (IO == kLdsToRegs) xio[r] = x[r];
            else lds[slot(r)] = x[r];
        }
    }
}

// a round of at most one group per thread with the table entries already in registers
template <int LOGN, int PRE, int P0, int S, RoundKind KIND, int LAZY, unsigned BIN, unsigned TOUT,
          RoundIo IO = kLdsToLds>
__device__ __forceinline__ void ntt_round_preloaded(uint64_t *lds, const RoundTable<S, KIND> &t,
                                                    const Mod &md, int tid, int h,
                                                    uint64_t *xio = nullptr)
{
    using Grp = Group<LOGN, P0, S>;
    if (tid >= (Grp::G >> PRE)) return;
    const Part part = part_of<LOGN, PRE, S>(h);
    const Grp grp(part.group0 + tid);
    uint64_t x[Grp::R];
    const int p0 = pad(grp.base - part.index0);
    auto slot = [&](int r) {
        return Grp::kSeparable ? p0 + Grp::padded_step(r) : pad(grp.at(r) - part.index0);
    };
#pragma unroll
    for (int r = 0; r < Grp::R; ++r) x[r] = IO == kRegsToLds ? xio[r] : lds[slot(r)];
    group_butterflies<S, KIND, LAZY, BIN, TOUT>(
        x, md, [&](int st, int j) { return t.f[(1 << st) - 1 + j]; },
        [&](int st, int j) { return t.i[(1 << st) - 1 + j]; }, [&](int r) { return t.s[r]; });
#pragma unroll
    for (int r = 0; r < Grp::R; ++r) {
        if constexpr (IO == kLdsToRegs) xio[r] = x[r];
        else lds[slot(r)] = x[r];
    }
}

// The rounds of a product by the secret over the stages PRE .. LOGN-1, in order: forward
// rounds 0 .. F-2, the round in the middle (last forward stages, pointwise product, first
// inverse stages), inverse rounds F-2 .. 0, F = rounds_for(LOGN - PRE, MAXS).
template <int LOGN, int PRE, int MAXS, int IDX>
struct RoundOf {
    static constexpr int F = rounds_for(LOGN - PRE, MAXS);
    static constexpr int TOTAL = 2 * F - 1;
    static constexpr int mirror(int idx) { return idx < F ? idx : 2 * F - 2 - idx; }   // forward round
    static constexpr int start_of(int j)
    {
        int p = PRE;
        for (int i = 0; i < j; ++i) p += round_stages(LOGN - p, MAXS);
        return p;
    }
    static constexpr int stages_of(int idx) { return round_stages(LOGN - start_of(mirror(idx)), MAXS); }
    static constexpr int J = mirror(IDX);
    static constexpr int P0 = start_of(J);
    static constexpr int S = stages_of(IDX);
    static constexpr RoundKind KIND = IDX == F - 1 ? kMiddle : (IDX < F ? kForward : kInverse);
    static constexpr int G = ((1 << LOGN) >> S) >> PRE;             // groups of one part
    // Lazy bounds of the rounds with inverse stages (idx >= F - 1), in multiples of q: what a
    // round folds behind its stages, and what its registers start from.
    static constexpr unsigned tout_of(int idx, int lazy)
    {
        return idx + 1 < TOTAL ? lazy_units(lazy) >> stages_of(idx + 1) : kFoldUnits;
    }
    static constexpr unsigned bin_of(int idx, int lazy)
    {
        unsigned b = product_units(lazy);                           // behind the pointwise product
        for (int i = F - 1; i < idx; ++i)
            b = inverse_round_out(stages_of(i), b, tout_of(i, lazy), product_units(lazy));
        return b;
    }
    static constexpr bool kInverseStages = IDX >= F - 1;
};

struct NoTable {};

// Stages per round by ring degree and batch size (see launch_poly): a batch that fills the
// chip several times runs 256 threads per polynomial where the ring allows it, a smaller one
// up to 1024.
constexpr int clamp_stages(int s) { return s < 2 ? 2 : (s > 4 ? 4 : s); }
constexpr int stages_large_batch(int logN) { return clamp_stages(logN - 8); }
constexpr int stages_small_batch(int logN) { return clamp_stages(logN - 10); }
// Table entries are asked for ahead of the barrier only in kernels that no large batch uses
// (a large batch hides the latency with other workgroups, and the registers cost it
// occupancy), only in rounds of at most two stages (3 to 10 entries), and only where a thread
// has a single group.
template <int LOGN, int PRE, int MAXS, int IDX, int NT>
constexpr bool preload_round()
{
    using Rd = RoundOf<LOGN, PRE, MAXS, IDX>;
    return PRE == 0 && MAXS == stages_small_batch(LOGN) && MAXS != stages_large_batch(LOGN) &&
           Rd::S <= 2 && Rd::G <= NT;
}

// The first and the last round can work from and to registers (see RoundIo) when the first
// round has one group per thread and there are rounds between them.
template <int LOGN, int PRE, int MAXS, int NT>
constexpr bool direct_ends()
{
    using First = RoundOf<LOGN, PRE, MAXS, 0>;
    return PRE == 0 && First::G == NT && First::TOTAL >= 3;
}

// Two consecutive rounds whose groups are 2^S coefficients at a stride of at most 64, one group
// per thread, keep every wave inside its own 64 * 2^S consecutive coefficients: wave w's 64
// groups are whole blocks of the round's first stage.  Between such rounds the workgroup need
// not meet: a wave's own LDS accesses complete in order.
template <int LOGN, int PRE, int MAXS, int IDX, int NT>
constexpr bool wave_local_after()
{
    using Me = RoundOf<LOGN, PRE, MAXS, IDX>;
    using Next = RoundOf<LOGN, PRE, MAXS, IDX + 1>;
    constexpr int lt_me = LOGN - Me::P0 - Me::S, lt_next = LOGN - Next::P0 - Next::S;
    return PRE == 0 && Me::S == Next::S && Me::G == NT && lt_me <= 6 && lt_next <= 6;
}
// what separates round IDX from round IDX + 1
template <int LOGN, int PRE, int MAXS, int IDX, int NT>
__device__ __forceinline__ void between_rounds()
{
    if constexpr (wave_local_after<LOGN, PRE, MAXS, IDX, NT>()) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        __syncthreads();
    }
}

// Round IDX and everything after it.  Where preload_round() says so, the next round's table
// entries are asked for before the barrier between the two rounds.
// `before_last()` runs in front of the last round: the caller asks there for what it needs from
// memory behind the product, and the round hides the latency.
// DIRECT: round 0 takes its coefficients from xio, the last round leaves its own there (below
// 2q) and no barrier follows it.
template <int LOGN, int PRE, int MAXS, int LAZY, bool DIRECT, int IDX, int NT, typename Table,
          typename Hook>
__device__ __forceinline__ void rounds_from(uint64_t *lds, const Twiddle *fwd, const Twiddle *inv,
                                            const Twiddle *shat, const Mod &md, int tid, int h,
                                            const Table &mine, Hook before_last, uint64_t *xio)
{
    using Me = RoundOf<LOGN, PRE, MAXS, IDX>;
    constexpr RoundIo IO = !DIRECT ? kLdsToLds
                                   : (IDX == 0 ? kRegsToLds : (IDX == Me::TOTAL - 1 ? kLdsToRegs : kLdsToLds));
    constexpr unsigned BIN = Me::kInverseStages ? Me::bin_of(IDX, LAZY) : 2u;
    constexpr unsigned TOUT = Me::kInverseStages ? Me::tout_of(IDX, LAZY) : 2u;
    if constexpr (IDX == Me::TOTAL - 1) before_last();
    if constexpr (preload_round<LOGN, PRE, MAXS, IDX, NT>())
        ntt_round_preloaded<LOGN, PRE, Me::P0, Me::S, Me::KIND, LAZY, BIN, TOUT, IO>(lds, mine, md, tid, h,
                                                                                   xio);
    else
        ntt_round<LOGN, PRE, Me::P0, Me::S, Me::KIND, NT, LAZY, BIN, TOUT, IO, true>(lds, fwd, inv, shat, md,
                                                                                   tid, h, xio);
    if constexpr (IDX + 1 < Me::TOTAL) {
        using Next = RoundOf<LOGN, PRE, MAXS, IDX + 1>;
        if constexpr (preload_round<LOGN, PRE, MAXS, IDX + 1, NT>()) {
            const int g = tid < Next::G ? tid : Next::G - 1;        // idle threads: any valid group
            const auto next = load_round_table<LOGN, Next::P0, Next::S, Next::KIND>(fwd, inv, shat, g);
            between_rounds<LOGN, PRE, MAXS, IDX, NT>();
            rounds_from<LOGN, PRE, MAXS, LAZY, DIRECT, IDX + 1, NT>(lds, fwd, inv, shat, md, tid, h, next,
                                                                    before_last, xio);
        } else {
            between_rounds<LOGN, PRE, MAXS, IDX, NT>();
            rounds_from<LOGN, PRE, MAXS, LAZY, DIRECT, IDX + 1, NT>(lds, fwd, inv, shat, md, tid, h,
                                                                    NoTable{}, before_last, xio);
        }
    } else if constexpr (!DIRECT) {
        __syncthreads();
    }
}

// The part times the secret (stages PRE .. LOGN-1 and back).
// Not DIRECT: the part is in the LDS and the caller has not yet passed the barrier behind its
// own writes (the first round's table entries are asked for in front of it); ends with a
// barrier, values below 2q in the LDS.
// DIRECT: thread `tid` brings coefficient tid + i NT in xio[i] and finds the product there
// afterwards, below 2q.
template <int LOGN, int PRE, int MAXS, int LAZY, bool DIRECT, int NT, typename Hook>
__device__ __forceinline__ void multiply_by_secret(uint64_t *lds, const Twiddle *fwd,
                                                   const Twiddle *inv, const Twiddle *shat,
                                                   const Mod &md, int tid, int h, Hook before_last,
                                                   uint64_t *xio)
{
    using First = RoundOf<LOGN, PRE, MAXS, 0>;
    if constexpr (preload_round<LOGN, PRE, MAXS, 0, NT>()) {
        const int g = tid < First::G ? tid : First::G - 1;
        const auto first = load_round_table<LOGN, First::P0, First::S, First::KIND>(fwd, inv, shat, g);
        if constexpr (!DIRECT) __syncthreads();
        rounds_from<LOGN, PRE, MAXS, LAZY, DIRECT, 0, NT>(lds, fwd, inv, shat, md, tid, h, first,
                                                          before_last, xio);
    } else {
        if constexpr (!DIRECT) __syncthreads();
        rounds_from<LOGN, PRE, MAXS, LAZY, DIRECT, 0, NT>(lds, fwd, inv, shat, md, tid, h, NoTable{},
                                                          before_last, xio);
    }
}

// forward stages P0 .. LOGN-1 of the part in the LDS; ends with a barrier
template <int LOGN, int PRE, int MAXS, int P0, int NT>
__device__ __forceinline__ void forward_only(uint64_t *lds, const Twiddle *fwd, const Mod &md, int tid,
                                             int h)
{
    if constexpr (P0 < LOGN) {
        constexpr int S = round_stages(LOGN - P0, MAXS);
        ntt_round<LOGN, PRE, P0, S, kForward, NT>(lds, fwd, nullptr, nullptr, md, tid, h);
        __syncthreads();
        forward_only<LOGN, PRE, MAXS, P0 + S, NT>(lds, fwd, md, tid, h);
    }
}

// the first PRE (0 or 1) forward stages on a pair (u, v) of coefficients N/2 apart: what part h
// of the ring starts from.  u, v < q; result below 3q.
template <int PRE>
__device__ __forceinline__ uint64_t enter_part(uint64_t u, uint64_t v, const Twiddle &w0, const Mod &md,
                                               int h)
{
    static_assert(PRE == 1, "one stage ahead of the parts");
    const uint64_t wv = mul_lazy(v, w0, md.nq);             // [0, 2q)
    return h == 0 ? u + wv : u + md.two_q - wv;
}

// ---------------------------------------------------------------------------
// c1 * s per (ciphertext, limb), then either the phase or the assembly of c0
// ---------------------------------------------------------------------------
struct PolyArgs {
    const Twiddle *tables;
    int set;        // table set of the product kernel that is launched (1 or 2)
    int L;
    // phase: src = ct [T][2][L][N], dst = phi [T][L][N]
    // encrypt: src = a [rows][L][N], dst = ctW [rows][2][L][N]
    const uint64_t *src;
    uint64_t *dst;
    // encrypt only
    const uint64_t *W;      // [k][n]
    const int8_t *e;        // [rows][N]
    int n, Ch;
    RlweArgs limbs;
};

// what becomes of coefficient c of the product as = (c1 or a) * s, as < q
__device__ __forceinline__ uint64_t finish_phase(uint64_t as, uint64_t c0, uint64_t q)
{
    const uint64_t v = as + c0;
    return v >= q ? v - q : v;
}

// Eq. (2) with chunking: coefficient c of chunk ch is column ch N + c, zero past n
__device__ __forceinline__ uint64_t encrypt_weight(const PolyArgs &a, uint32_t row, uint32_t c, int N)
{
    const uint32_t i = row / (uint32_t)a.Ch, ch = row % (uint32_t)a.Ch;
    const uint32_t col = ch * (uint32_t)N + c;
    return col < (uint32_t)a.n ? a.W[(size_t)i * a.n + col] : 0;
}
// c0 = Delta w + e - a s  for the weight w and the error ev of the coefficient, as < q
__device__ __forceinline__ uint64_t finish_encrypt(uint64_t as, uint64_t w, int ev, const RlweLimb &P)
{
    const uint64_t q = P.red.q;
    uint64_t v = barrett128(__umul64hi(P.delta, w), P.delta * w, P.red);       // w < t < q
    v += ev < 0 ? q - (uint64_t)(-ev) : (uint64_t)ev;
    v += q - as;                                // < 3q
    v = v >= q ? v - q : v;
    return v >= q ? v - q : v;
}

// PRE = 0: the whole product and what follows it in one kernel.  PRE = 1 (ring of 2^15
// coefficients): workgroup (polynomial, h) does part h: first forward stage on the way in,
// stages 1 .. LOGN-1 and back in the LDS, and leaves its half of the not yet joined product
// where the result will be (phi, or the c0 half of the ciphertext); rlwe_join_kernel does
// the last inverse stage and what follows.
// LAZY: kLoose where every modulus of the call lies in [2^34, 2^58), kTight where in [2^34, 2^59),
// else kNever (see group_butterflies).
template <int LOGN, int PRE, int MAXS, bool ENCRYPT, int LAZY>
__global__ __launch_bounds__(threads_for(LOGN - PRE, MAXS)) void rlwe_poly_kernel(PolyArgs a)
{
    constexpr int N = 1 << LOGN, NP = N >> PRE, NT = threads_for(LOGN - PRE, MAXS);
    __shared__ uint64_t lds[padded_size(NP)];
    const int tid = threadIdx.x;
    const uint32_t poly = blockIdx.x >> PRE;
    const int h = (int)(blockIdx.x & ((1u << PRE) - 1u));
    const uint32_t row = poly / (uint32_t)a.L, l = poly % (uint32_t)a.L;
    const RlweLimb &P = a.limbs.limb[l];
    const uint64_t q = P.red.q;
    const Mod md = make_mod(P);
    const Twiddle *const t = a.tables + (size_t)l * limb_table_entries(N) + (size_t)a.set * set_entries(N);
    // the polynomial that is multiplied by s
    const uint64_t *const mul_in =
        ENCRYPT ? a.src + ((size_t)row * a.L + l) * N
                : a.src + (((size_t)row * 2 + 1) * a.L + l) * N;
    // where the result goes: phi[row][l], or c0 of ciphertext `row`
    uint64_t *const out = ENCRYPT ? a.dst + (((size_t)row * 2 + 0) * a.L + l) * N
                                  : a.dst + ((size_t)row * a.L + l) * N;
    // c1 = a is copied while a is on its way into the LDS (one read of a in all)
    uint64_t *const c1 = a.dst + (((size_t)row * 2 + 1) * a.L + l) * N;
    // Coefficient mine(i) of the part is this thread's on the way in and on the way out.  All
    // the loads of a pass are issued before the first of them is waited for.
    constexpr int IT = (NP + NT - 1) / NT;
    constexpr bool kRagged = NP % NT != 0;          // rings below the 64 threads of a wave
    constexpr bool DIRECT = direct_ends<LOGN, PRE, MAXS, NT>();
    auto mine = [&](int i) { return tid + i * NT; };
    auto have = [&](int i) { return !kRagged || mine(i) < NP; };
    uint64_t x[IT];                                 // DIRECT: in and out of the product
    if constexpr (PRE == 0) {
#pragma unroll
        for (int i = 0; i < IT; ++i) x[i] = have(i) ? mul_in[mine(i)] : 0;
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            if (!have(i)) continue;
            if constexpr (!DIRECT) lds[pad(mine(i))] = x[i];
            if constexpr (ENCRYPT) c1[mine(i)] = x[i];
        }
    } else {
        const Twiddle w0 = t[1];
        uint64_t v[IT];
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            x[i] = have(i) ? mul_in[mine(i)] : 0;
            v[i] = have(i) ? mul_in[mine(i) + NP] : 0;
        }
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            if (!have(i)) continue;
            lds[pad(mine(i))] = enter_part<PRE>(x[i], v[i], w0, md, h);
            if constexpr (ENCRYPT) c1[h * NP + mine(i)] = h == 0 ? x[i] : v[i];
        }
    }
    // what is added to the product: c0 (phase), or the weight and the error (encryption);
    // asked for in front of the last round
    uint64_t addend[IT];
    int err[IT];
    auto before_last = [&]() {
        if constexpr (PRE == 0) {
#pragma unroll
            for (int i = 0; i < IT; ++i) {
                if constexpr (ENCRYPT) {
                    addend[i] = have(i) ? encrypt_weight(a, row, (uint32_t)mine(i), N) : 0;
                    err[i] = have(i) ? a.e[(size_t)row * N + mine(i)] : 0;
                } else {
                    addend[i] = have(i) ? a.src[(((size_t)row * 2 + 0) * a.L + l) * N + mine(i)] : 0;
                }
            }
        }
    };
    multiply_by_secret<LOGN, PRE, MAXS, LAZY, DIRECT, NT>(lds, t, t + N, t + 2 * N, md, tid, h, before_last,
                                                          x);
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        if (!have(i)) continue;
        const uint64_t as = cond_sub(DIRECT ? x[i] : lds[pad(mine(i))], md.nq);     // [0, 2q) -> [0, q)
        if constexpr (PRE != 0) {
            out[h * NP + mine(i)] = as;
        } else if constexpr (ENCRYPT) {
            out[mine(i)] = finish_encrypt(as, addend[i], err[i], P);
        } else {
            out[mine(i)] = finish_phase(as, addend[i], q);
        }
    }
}

// Last inverse stage of a ring handled in two parts, in place on the two halves the part
// kernels left in `out`: (u, v) -> (u + v, (u - v) psi^-brv(1)), then what follows the
// product.  One thread per pair of coefficients N/2 apart.
template <bool ENCRYPT>
__global__ __launch_bounds__(256) void rlwe_join_kernel(PolyArgs a, int logN, uint64_t pairs)
{
    const uint64_t gid = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (gid >= pairs) return;
    const int N = 1 << logN, NP = N >> 1;
    const uint32_t poly = (uint32_t)(gid >> (logN - 1)), c = (uint32_t)(gid & (uint64_t)(NP - 1));
    const uint32_t row = poly / (uint32_t)a.L, l = poly % (uint32_t)a.L;
    const RlweLimb &P = a.limbs.limb[l];
    const uint64_t q = P.red.q;
    const Twiddle w0_inv = a.tables[(size_t)l * limb_table_entries(N) + N + 1];
    uint64_t *const out = ENCRYPT ? a.dst + (((size_t)row * 2 + 0) * a.L + l) * N
                                  : a.dst + ((size_t)row * a.L + l) * N;
    const uint64_t u = out[c], v = out[c + NP];             // < q
    uint64_t lo = u + v;
    lo = lo >= q ? lo - q : lo;
    uint64_t hi = mul_lazy(u + q - v, w0_inv, 0 - q);       // [0, 2q)
    hi = hi >= q ? hi - q : hi;
    if constexpr (ENCRYPT) {
        out[c] = finish_encrypt(lo, encrypt_weight(a, row, c, N), a.e[(size_t)row * N + c], P);
        out[c + NP] = finish_encrypt(hi, encrypt_weight(a, row, c + NP, N), a.e[(size_t)row * N + c + NP], P);
    } else {
        const uint64_t *const c0 = a.src + (((size_t)row * 2 + 0) * a.L + l) * N;
        out[c] = finish_phase(lo, c0[c], q);
        out[c + NP] = finish_phase(hi, c0[c + NP], q);
    }
}

#define NIMBUS_RLWE_DISPATCH(logN, CALL)                                          \
    switch (logN) {                                                               \
    case 5: { constexpr int LOGN = 5; return CALL; }                              \
    case 6: { constexpr int LOGN = 6; return CALL; }                              \
    case 7: { constexpr int LOGN = 7; return CALL; }                              \
    case 8: { constexpr int LOGN = 8; return CALL; }                              \
    case 9: { constexpr int LOGN = 9; return CALL; }                              \
    case 10: { constexpr int LOGN = 10; return CALL; }                            \
    case 11: { constexpr int LOGN = 11; return CALL; }                            \
    case 12: { constexpr int LOGN = 12; return CALL; }                            \
    case 13: { constexpr int LOGN = 13; return CALL; }                            \
    case 14: { constexpr int LOGN = 14; return CALL; }                            \
    default: return hipErrorInvalidValue;                                         \
    }

// Table sets: 1 for the kernels of large batches (and the ring of 2^15), 2 for small batches.
constexpr int kSetLargeBatch = 1, kSetSmallBatch = 2;

// which of the kernels applies: without conditional subtractions where every modulus leaves
// the room (see group_butterflies)
static int lazy_kind(const PolyArgs &a)
{
    int kind = kLoose;
    for (int l = 0; l < a.L; ++l) {
        const uint64_t q = a.limbs.limb[l].red.q;
        if (q < (1ull << 34) || q >= (1ull << 59)) return kNever;
        if (q >= (1ull << 58)) kind = kTight;
    }
    return kind;
}

template <bool ENCRYPT, int MAXS, int LAZY>
static hipError_t launch_poly_with(const PolyArgs &a, int logN, size_t polys, hipStream_t stream)
{
    NIMBUS_RLWE_DISPATCH(logN, launch(rlwe_poly_kernel<LOGN, 0, MAXS, ENCRYPT, LAZY>, dim3((unsigned)polys),
                                      dim3(threads_for(LOGN, MAXS)), stream, a));
}
template <bool ENCRYPT, int MAXS>
static hipError_t launch_poly_stages(const PolyArgs &a, int logN, size_t polys, hipStream_t stream)
{
    switch (lazy_kind(a)) {
    case kLoose: return launch_poly_with<ENCRYPT, MAXS, kLoose>(a, logN, polys, stream);
    case kTight: return launch_poly_with<ENCRYPT, MAXS, kTight>(a, logN, polys, stream);
    default: return launch_poly_with<ENCRYPT, MAXS, kNever>(a, logN, polys, stream);
    }
}

// ring of 2^15 coefficients: two workgroups per polynomial, then the joining pass
template <bool ENCRYPT>
static hipError_t launch_poly_in_parts(PolyArgs a, size_t polys, hipStream_t stream)
{
    a.set = kSetLargeBatch;
    const dim3 grid(2u * (unsigned)polys), block(threads_for(14, 4));
    hipError_t e;
    switch (lazy_kind(a)) {
    case kLoose: e = launch(rlwe_poly_kernel<15, 1, 4, ENCRYPT, kLoose>, grid, block, stream, a); break;
    case kTight: e = launch(rlwe_poly_kernel<15, 1, 4, ENCRYPT, kTight>, grid, block, stream, a); break;
    default: e = launch(rlwe_poly_kernel<15, 1, 4, ENCRYPT, kNever>, grid, block, stream, a); break;
    }
    if (e != hipSuccess) return e;
    const uint64_t pairs = (uint64_t)polys << 14;
    return launch(rlwe_join_kernel<ENCRYPT>, dim3((unsigned)((pairs + 255u) / 256u)), dim3(256),
                  stream, a, 15, pairs);
}

// Stages per round by ring degree and batch size (one workgroup per polynomial, 256 compute
// units).  A batch that fills the chip several times runs 256 threads per polynomial where
// the ring allows it (several workgroups per compute unit hide each other's latencies); a
// smaller batch runs up to 1024 threads per polynomial, because then one workgroup has the
// compute unit to itself and its own waves are all there is to overlap.
template <bool ENCRYPT>
static hipError_t launch_poly(PolyArgs a, int logN, size_t polys, hipStream_t stream)
{
    if (logN == 15) return launch_poly_in_parts<ENCRYPT>(a, polys, stream);
    const bool large = polys >= 1024;
    const int maxs = large ? stages_large_batch(logN) : stages_small_batch(logN);
    a.set = large ? kSetLargeBatch : kSetSmallBatch;
    if (maxs == 4) return launch_poly_stages<ENCRYPT, 4>(a, logN, polys, stream);
    if (maxs == 3) return launch_poly_stages<ENCRYPT, 3>(a, logN, polys, stream);
    return launch_poly_stages<ENCRYPT, 2>(a, logN, polys, stream);
}

// the encryption's launches (rlwe_encrypt.hip)
hipError_t launch_encrypt_rows(const PolyArgs &a, int logN, size_t polys, hipStream_t stream);

}  // namespace nimbus
