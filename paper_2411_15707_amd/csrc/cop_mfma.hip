// Matrix-core (int8 MFMA) kernels for the COP accumulation, gfx950.
//
// The contraction out = X * ctW (Algorithm 1 step 2 of the paper) is an exact
// integer matrix product with a 2^x_bits-bounded left operand and a q-bounded
// right operand.  Both are split into signed bytes so that the products run on
// v_mfma_i32_32x32x32_i8:
//
//   x  = x' + OFFX,  x' = sum_{a<DX} dx_a 256^a,  dx_a = byte_a(x) - 128,
//                    OFFX = sum_{a<DX} 128 * 256^a            (no carries needed)
//   c' = c or c - q  (centred, |c'| <= (q-1)/2),  c' = sum_{b<DQ} dq_b 256^b,
//                    dq_b in [-128, 127]  (carry-propagating recode, done once
//                    per weight matrix by nimbus_cop_prepare)
//
//   sum_i x_i c_i  =  sum_i x'_i c'_i  +  OFFX * S   (mod q),   S = sum_i c_i mod q
//   sum_i x'_i c'_i = sum_d 256^d D_d,   D_d = sum_{a+b=d} sum_i dx_a(i) dq_b(i)
//
// Each D_d is one int32 MFMA accumulator (all byte pairs of one diagonal d
// accumulate into the same tile).  |dx dq| <= 2^14, at most min(DX,DQ) pairs per
// diagonal, so |D_d| <= k * min(DX,DQ) * 2^14, which the host keeps below 2^30.
// The accumulators start at 2^30, so what comes out is D_d + 2^30 in [0, 2^31):
// the epilogue rebuilds sum_d (D_d + 2^30) 256^d with unsigned 32-bit pieces, adds
// one 128-bit constant (a multiple of q that makes the total non-negative, plus
// OFFX*S, minus the 2^30 offsets), adds the mask, and reduces once.
//
// Operand tiles are 32 x 32 bytes stored in the register order of the MFMA: the
// 16 bytes of lane l belong to row (or column) l % 32 and to k-slots
// (l / 32) * 16 .. +15 of the tile.  The A and B operands of the instruction
// use the same lane/byte -> k mapping, so any fixed assignment of k-slots to
// actual k indices gives the same sum as long as both sides share it.
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
// setup phase: canonical ctW -> signed byte planes of the centred residues
// one thread fills the 16 bytes of one lane slot in each of the DQ planes of a tile
// ---------------------------------------------------------------------------
template <int DQ>
__global__ __launch_bounds__(256) void prepare_planes_kernel(
    const uint64_t *__restrict__ ctW, int k, uint32_t C, int N, int L, LimbTable limbs,
    int KB, uint64_t total, uint4 *__restrict__ planes)
{
    const uint64_t gid = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (gid >= total) return;
    const uint32_t lane = (uint32_t)(gid & 63u);
    const uint64_t tile = gid >> 6;                 // ct * KB + kb
    const uint32_t kb = (uint32_t)(tile % (uint64_t)KB);
    const uint32_t ct = (uint32_t)(tile / (uint64_t)KB);
    const uint32_t col = ct * kTile + (lane & 31u);
    const int kbase = (int)kb * kTile + (int)(lane >> 5) * 16;
    const uint64_t q = limbs.limb[(col / (uint32_t)N) % (uint32_t)L].q;
    const uint64_t half = (q - 1) >> 1;

    uint64_t bias = 0;                              // 0x80 in each of the DQ low bytes
#pragma unroll
    for (int d = 0; d < DQ; ++d) bias |= (uint64_t)0x80 << (8 * d);

    uint32_t w[DQ][4];
#pragma unroll
    for (int d = 0; d < DQ; ++d) { w[d][0] = w[d][1] = w[d][2] = w[d][3] = 0; }

#pragma unroll
    for (int b = 0; b < 16; ++b) {
        const int i = kbase + b;
        if (i < k) {
            const uint64_t c = ctW[(size_t)i * C + col];
            const uint64_t cc = c > half ? c - q : c;          // two's complement of c'
            // c' + bias has unsigned bytes dq_b + 128; flipping bit 7 gives dq_b as int8
            const uint64_t v = (cc + bias) ^ bias;
#pragma unroll
            for (int d = 0; d < DQ; ++d)
                w[d][b >> 2] |= (uint32_t)((v >> (8 * d)) & 0xffu) << (8 * (b & 3));
        }
    }
#pragma unroll
    for (int d = 0; d < DQ; ++d)
        planes[(tile * DQ + d) * 64u + lane] = make_uint4(w[d][0], w[d][1], w[d][2], w[d][3]);
}

// S[col] = sum_i ctW[i][col] mod q
__global__ __launch_bounds__(256) void column_sums_kernel(
    const uint64_t *__restrict__ ctW, int k, uint32_t C, int N, int L, LimbTable limbs,
    uint64_t *__restrict__ colsum)
{
    const uint32_t col = blockIdx.x * 256u + threadIdx.x;
    if (col >= C) return;
    const Limb P = limbs.limb[(col / (uint32_t)N) % (uint32_t)L];
    uint64_t hi = 0, lo = 0;
    for (int i = 0; i < k; ++i) add128(hi, lo, 0, ctW[(size_t)i * C + col]);
    colsum[col] = barrett128(hi, lo, P);            // k * q < 2^(b+63)
}

// ---------------------------------------------------------------------------
// per call: X -> DX signed byte planes in A-operand tile order
// ---------------------------------------------------------------------------
template <int DX>
__global__ __launch_bounds__(256) void x_planes_kernel(
    const uint64_t *__restrict__ X, int m, int k, int KB, uint32_t total,
    uint4 *__restrict__ xd)
{
    const uint32_t gid = blockIdx.x * 256u + threadIdx.x;
    if (gid >= total) return;
    const uint32_t lane = gid & 63u;
    const uint32_t tile = gid >> 6;                 // rt * KB + kb
    const uint32_t kb = tile % (uint32_t)KB;
    const uint32_t rt = tile / (uint32_t)KB;
    const int row = (int)rt * kTile + (int)(lane & 31u);
    const int kbase = (int)kb * kTile + (int)(lane >> 5) * 16;

    uint32_t w[DX][4];
#pragma unroll
    for (int d = 0; d < DX; ++d) { w[d][0] = w[d][1] = w[d][2] = w[d][3] = 0; }
    if (row < m) {
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            const int i = kbase + b;
            if (i < k) {
                const uint32_t x = (uint32_t)X[(size_t)row * k + i] ^ 0x80808080u;
#pragma unroll
                for (int d = 0; d < DX; ++d)
                    w[d][b >> 2] |= ((x >> (8 * d)) & 0xffu) << (8 * (b & 3));
            }
        }
    }
#pragma unroll
    for (int d = 0; d < DX; ++d)
        xd[((size_t)tile * DX + d) * 64u + lane] = make_uint4(w[d][0], w[d][1], w[d][2], w[d][3]);
}

// ---------------------------------------------------------------------------
// main kernel
// workgroup = 4 waves = 128 token rows x one 32-column tile; wave w owns the
// 32 x 32 output tile of rows rb*128 + w*32 .. +31 with DX+DQ-1 accumulators.
// B (ciphertext planes) streams global -> LDS in stages of KS k-blocks, double
// buffered; A (X planes, L2 resident) is read straight into registers.
// ---------------------------------------------------------------------------
struct MfmaArgs {
    const uint4 *xd;          // [RT][KB][DX][64] uint4
    const uint4 *planes;      // [CT][KB][DQ][64] uint4
    const uint64_t *colsum;   // [C]
    const uint64_t *mask;     // [m][C] or null
    uint64_t *out;            // [m][C]
    int m, KB, RB, N, L;
    uint32_t C, CT;
    uint32_t offx;            // OFFX
    uint64_t q[kMaxLimbs];
    double qinv[kMaxLimbs];   // 1 / q_l, rounded
    // (q_l << sh) - 2^30 * sum_d 256^d  modulo 2^128
    uint64_t cst_hi[kMaxLimbs], cst_lo[kMaxLimbs];
};

// V mod q for 0 <= V = hi:lo < 2^47 * q, q < 2^62.
// The quotient is estimated in double precision: V converted with three roundings, times
// the rounded 1/q, has a relative error below 2^-50, so below 2^47 the estimate is off
// by less than 1/8; taking 1/4 off before truncating gives floor(V/q) or one less,
// never more.  The remainder is then formed modulo 2^64 and corrected once.
__device__ __forceinline__ uint64_t reduce_fp(uint64_t hi, uint64_t lo, uint64_t q, double qinv)
{
    const double two32 = 4294967296.0;
    double vd = fma((double)(uint32_t)(lo >> 32), two32, (double)(uint32_t)lo);
    vd = fma((double)(uint32_t)hi, two32 * two32, vd);
    vd = fma((double)(uint32_t)(hi >> 32), two32 * two32 * two32, vd);
    const double qd = fmax(fma(vd, qinv, -0.25), 0.0);
    const uint32_t qh = (uint32_t)(qd * (1.0 / two32));
    const uint32_t ql = (uint32_t)fma(-(double)qh, two32, qd);
    const uint32_t q_lo = (uint32_t)q, q_hi = (uint32_t)(q >> 32);
    uint64_t p = (uint64_t)ql * q_lo;
    p += (uint64_t)(ql * q_hi + qh * q_lo) << 32;
    uint64_t r = lo - p;
    if (r >= q) r -= q;
    return r;
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

// wait until at most PENDING of this wave's global loads (here: direct-to-LDS loads) are
// outstanding
template <int PENDING>
__device__ __forceinline__ void wait_vmem()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PENDING) : "memory");
}

// one wave copies 64 x 16 B (a whole operand tile) or 64 x 4 B (a quarter tile) from
// global memory straight into LDS; lane l's bytes land at dst + l*16 (resp. l*4)
__device__ __forceinline__ void dma_tile(const void *src_lane, void *dst_wave)
{
    __builtin_amdgcn_global_load_lds((const NIMBUS_AS1 void *)src_lane,
                                     (NIMBUS_AS3 void *)dst_wave, 16, 0, 0);
}
__device__ __forceinline__ void dma_quarter(const void *src_lane, void *dst_wave)
{
    __builtin_amdgcn_global_load_lds((const NIMBUS_AS1 void *)src_lane,
                                     (NIMBUS_AS3 void *)dst_wave, 4, 0, 0);
}

// The pipeline: a stage is one k-block (32 values of k): the workgroup's 4*DX operand
// tiles of X and the DQ operand tiles of the ciphertext planes, STAGE_TILES KB in all.
// Stages live in a ring of RING LDS buffers filled by direct-to-LDS loads issued
// RING-1 stages ahead; nothing passes through registers on the way in.  Every wave
// issues the same number of loads per stage (its own DX tiles of X, one whole ciphertext
// tile, and a quarter of each remaining ciphertext tile), so "stage s has landed" is the
// wait "at most (stages issued after s) * LOADS loads pending" followed by the barrier.
template <int DX, int DQ>
struct Pipe {
    static constexpr int A_TILES = 4 * DX;
    static constexpr int STAGE_TILES = A_TILES + DQ;
    static constexpr int STAGE_BYTES = STAGE_TILES * kTileBytes;
    static constexpr int RING = (4 * STAGE_BYTES <= 80 * 1024) ? 4 : 3;
    static constexpr int LOADS = DX + 1 + (DQ - 4);
    static_assert(DQ >= 4, "each of the four waves moves one whole ciphertext tile");
};

template <int DX, int DQ>
__global__ __launch_bounds__(256, 2) void cop_mfma_kernel(const MfmaArgs a)
{
    using P_ = Pipe<DX, DQ>;
    constexpr int ND = DX + DQ - 1;
    constexpr int RING = P_::RING;
    constexpr int LOADS = P_::LOADS;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[RING * P_::STAGE_BYTES];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // workgroup -> (column tile, row block).  Workgroups are dealt round-robin to
    // the 8 XCDs; the RB row blocks that share a column tile are kept on one XCD
    // and adjacent in launch order so that tile is fetched from HBM once.
    uint32_t ct, rb;
    {
        const uint32_t id = blockIdx.x;
        if ((a.CT & 7u) == 0) {
            const uint32_t xcd = id & 7u, slot = id >> 3;
            rb = slot % (uint32_t)a.RB;
            ct = (slot / (uint32_t)a.RB) * 8u + xcd;
        } else {
            rb = id % (uint32_t)a.RB;
            ct = id / (uint32_t)a.RB;
        }
    }
    const int rt = (int)rb * 4 + wave;
    const bool active = rt * kTile < a.m;           // wave-uniform
    // a wave without rows still moves its share of every stage (reading the last real
    // row tile in place of its own) so that all waves count the same loads
    const int rt_load = active ? rt : (a.m - 1) / kTile;

    const int KB = a.KB;
    const unsigned char *gA = (const unsigned char *)(a.xd + (size_t)rt_load * KB * (DX * 64));
    const unsigned char *gB = (const unsigned char *)(a.planes + (size_t)ct * KB * (DQ * 64));

    auto issue = [&](int kb, int buf) {
        unsigned char *dst = lds + buf * P_::STAGE_BYTES;
        const unsigned char *srcA = gA + (size_t)kb * (DX * kTileBytes);
        const unsigned char *srcB = gB + (size_t)kb * (DQ * kTileBytes);
#pragma unroll
        for (int d = 0; d < DX; ++d)
            dma_tile(srcA + d * kTileBytes + lane * 16, dst + (wave * DX + d) * kTileBytes);
        dma_tile(srcB + wave * kTileBytes + lane * 16, dst + (P_::A_TILES + wave) * kTileBytes);
#pragma unroll
        for (int d = 4; d < DQ; ++d)
            dma_quarter(srcB + d * kTileBytes + wave * 256 + lane * 4,
                        dst + (P_::A_TILES + d) * kTileBytes + wave * 256);
    };

    v16i acc[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[d][r] = 1 << 30;

    // Operands come out of LDS through explicit ds_read_b128 instructions: reads the
    // compiler can see would each be made to wait for every direct-to-LDS load in
    // flight.  All reads of a k-block are issued at once; the matrix-core work on
    // ciphertext plane dq starts as soon as that plane is back.
    const uint32_t lds0 = (uint32_t)(uintptr_t)(NIMBUS_AS3 void *)&lds[0];
    const uint32_t laneA = lds0 + (uint32_t)(wave * DX) * kTileBytes + (uint32_t)lane * 16u;
    const uint32_t laneB = lds0 + (uint32_t)P_::A_TILES * kTileBytes + (uint32_t)lane * 16u;
    auto compute = [&](int buf) {
        const uint32_t off = (uint32_t)buf * P_::STAGE_BYTES;
        v4i xa[DX], b[DQ];
        static_for<0, DX>([&](auto d_c) {
            constexpr int d = decltype(d_c)::value;
            xa[d] = lds_read_b128<d * kTileBytes>(laneA + off);
        });
        static_for<0, DQ>([&](auto d_c) {
            constexpr int d = decltype(d_c)::value;
            b[d] = lds_read_b128<d * kTileBytes>(laneB + off);
        });
        static_for<0, DQ>([&](auto dq_c) {
            constexpr int dq = decltype(dq_c)::value;
            wait_lds<DQ - 1 - dq>(b[dq]);
            if constexpr (dq == 0) {
#pragma unroll
                for (int dx = 0; dx < DX; ++dx) asm volatile("" : "+v"(xa[dx]));
            }
#pragma unroll
            for (int dx = 0; dx < DX; ++dx)
                acc[dx + dq] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                    xa[dx], b[dq], acc[dx + dq], 0, 0, 0);
        });
    };

    // prologue: stages 0 .. RING-2
#pragma unroll
    for (int s = 0; s < RING - 1; ++s)
        if (s < KB) issue(s, s);
    asm volatile("" ::: "memory");

    for (int s = 0; s < KB; ++s) {
        // stages issued so far: 0 .. min(KB-1, s+RING-2); those after s are still allowed
        // to be in flight
        const int last = (s + RING - 2 < KB - 1) ? (s + RING - 2) : (KB - 1);
        const int younger = last - s;
        if (younger >= 2) wait_vmem<2 * LOADS>();
        else if (younger == 1) wait_vmem<LOADS>();
        else wait_vmem<0>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // every wave is past stage s-1: its buffer can take stage s+RING-1
        if (s + RING - 1 < KB) issue(s + RING - 1, (s + RING - 1) % RING);
        asm volatile("" ::: "memory");
        if (active) compute(s % RING);
    }
    if (!active) return;

    // ---- epilogue: rebuild, add the constant and the mask, reduce, store ----
    const uint32_t col = ct * kTile + (uint32_t)(lane & 31);
    const uint32_t limb = (ct * kTile / (uint32_t)a.N) % (uint32_t)a.L;   // uniform
    const uint64_t q = a.q[limb];
    const double qinv = a.qinv[limb];
    uint64_t cst_hi = a.cst_hi[limb], cst_lo = a.cst_lo[limb];
    {
        const uint64_t S = a.colsum[col];
        add128(cst_hi, cst_lo, __umul64hi(S, (uint64_t)a.offx), S * (uint64_t)a.offx);
    }
    const int row0 = rt * kTile + 4 * (lane >> 5);
    // all mask words first, so that their latencies overlap
    uint64_t mk[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = row0 + 8 * (r >> 2) + (r & 3);
        mk[r] = (a.mask && row < a.m) ? a.mask[(size_t)row * a.C + col] : 0;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = row0 + 8 * (r >> 2) + (r & 3);
        if (row < a.m) {
            // E_d = D_d + 2^30 < 2^31.  Z_b = E_b + 2^32 E_{b+4} is a register pair;
            // sum_d E_d 256^d = Z_0 + 2^8 Z_1 + 2^16 Z_2 + 2^24 Z_3 + 2^64 (E_8 + ...)
            auto E = [&](int d) -> uint64_t { return d < ND ? (uint64_t)(uint32_t)acc[d][r] : 0; };
            uint64_t lo = E(0) | (E(4) << 32);
            uint64_t hi = E(8) + (E(9) << 8) + (E(10) << 16);
#pragma unroll
            for (int b = 1; b < 4; ++b) {
                const uint64_t Z = E(b) | (E(b + 4) << 32);
                const uint64_t t = Z << (8 * b);
                lo += t;
                hi += (Z >> (64 - 8 * b)) + (lo < t ? 1u : 0u);
            }
            add128(hi, lo, cst_hi, cst_lo);
            add128(hi, lo, 0, mk[r]);
            a.out[(size_t)row * a.C + col] = reduce_fp(hi, lo, q, qinv);
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static int ceil_log2(unsigned v)
{
    int b = 0;
    while ((1ull << b) < v) ++b;
    return b;
}

// q * 2^sh is added to make the signed sum non-negative: 2^sh >= k * 2^(8 DX - 1)
// bounds |sum_i x'_i c'_i| / q from above (|x'| < 2^(8 DX - 1) * 1.01, |c'| <= q / 2)
static int bias_shift(const Problem &p)
{
    return ceil_log2((unsigned)p.k) + 8 * planes_x(p.x_bits) - 1;
}

bool mfma_supported(const Problem &p)
{
    const int DX = planes_x(p.x_bits), DQ = planes_q(p.q_bits_max);
    if (DX < 2 || DX > 4 || DQ < 7 || DQ > 8) return false;
    const long long pairs = DX < DQ ? DX : DQ;
    // |D_d| < 2^30 (zero padding of k adds nothing)
    if ((long long)p.k * pairs * 16384ll >= (1ll << 30)) return false;
    // the value reduced in the epilogue is below (2^(sh+1) + 2^32 + 1) * q; the
    // floating-point quotient needs it below 2^47 * q
    return bias_shift(p) + 2 <= 47;
}

template <int DQ>
static hipError_t prepare_impl(const Problem &p, const uint64_t *ctW, void *prepared,
                               hipStream_t stream)
{
    const int KB = kblocks(p.k);
    const uint32_t CT = (uint32_t)(p.C / kTile);
    const uint64_t total = (uint64_t)CT * KB * 64;
    uint4 *planes = (uint4 *)prepared;
    uint64_t *colsum = (uint64_t *)((char *)prepared + (size_t)CT * KB * DQ * kTileBytes);
    hipLaunchKernelGGL(prepare_planes_kernel<DQ>, dim3((unsigned)((total + 255) / 256)), dim3(256),
                       0, stream, ctW, p.k, (uint32_t)p.C, p.N, p.L, p.limbs, KB, total, planes);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(column_sums_kernel, dim3((unsigned)((p.C + 255) / 256)), dim3(256), 0,
                       stream, ctW, p.k, (uint32_t)p.C, p.N, p.L, p.limbs, colsum);
    return hipGetLastError();
}

hipError_t launch_prepare(const Problem &p, const uint64_t *ctW, void *prepared,
                          hipStream_t stream)
{
    if (planes_q(p.q_bits_max) == 7) return prepare_impl<7>(p, ctW, prepared, stream);
    return prepare_impl<8>(p, ctW, prepared, stream);
}

template <int DX>
static hipError_t stage_impl(const Problem &p, const uint64_t *X, void *workspace,
                             hipStream_t stream)
{
    const int KB = kblocks(p.k);
    const int RT = (p.m + kTile - 1) / kTile;
    const uint32_t xtotal = (uint32_t)RT * KB * 64;
    hipLaunchKernelGGL(x_planes_kernel<DX>, dim3((xtotal + 255) / 256), dim3(256), 0, stream,
                       X, p.m, p.k, KB, xtotal, (uint4 *)workspace);
    return hipGetLastError();
}

hipError_t launch_stage_shares(const Problem &p, const uint64_t *X, void *workspace,
                               hipStream_t stream)
{
    switch (planes_x(p.x_bits)) {
    case 2: return stage_impl<2>(p, X, workspace, stream);
    case 3: return stage_impl<3>(p, X, workspace, stream);
    default: return stage_impl<4>(p, X, workspace, stream);
    }
}

template <int DX, int DQ>
static hipError_t mfma_impl(const Problem &p, const void *staged, const void *prepared,
                            const uint64_t *mask, uint64_t *out, hipStream_t stream)
{
    const int KB = kblocks(p.k);
    const uint32_t CT = (uint32_t)(p.C / kTile);

    MfmaArgs a{};
    a.xd = (const uint4 *)staged;
    a.planes = (const uint4 *)prepared;
    a.colsum = (const uint64_t *)((const char *)prepared + (size_t)CT * KB * DQ * kTileBytes);
    a.mask = mask;
    a.out = out;
    a.m = p.m;
    a.KB = KB;
    a.RB = (p.m + 127) / 128;
    a.N = p.N;
    a.L = p.L;
    a.C = (uint32_t)p.C;
    a.CT = CT;
    a.offx = 0;
    for (int d = 0; d < DX; ++d) a.offx |= 0x80u << (8 * d);
    const int sh = bias_shift(p);
    unsigned __int128 offsets = 0;                  // 2^30 * sum_d 256^d
    for (int d = 0; d < DX + DQ - 1; ++d) offsets += (unsigned __int128)1 << (30 + 8 * d);
    for (int l = 0; l < p.L; ++l) {
        const uint64_t q = p.limbs.limb[l].q;
        const unsigned __int128 c = ((unsigned __int128)q << sh) - offsets;   // modulo 2^128
        a.q[l] = q;
        a.qinv[l] = 1.0 / (double)q;
        a.cst_hi[l] = (uint64_t)(c >> 64);
        a.cst_lo[l] = (uint64_t)c;
    }
    hipLaunchKernelGGL((cop_mfma_kernel<DX, DQ>), dim3(CT * (uint32_t)a.RB), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_cop_mfma(const Problem &p, const void *staged, const void *prepared,
                           const uint64_t *mask, uint64_t *out, hipStream_t stream)
{
    const int DX = planes_x(p.x_bits), DQ = planes_q(p.q_bits_max);
#define NIMBUS_CASE(dx, dq) \
    if (DX == dx && DQ == dq) return mfma_impl<dx, dq>(p, staged, prepared, mask, out, stream);
    NIMBUS_CASE(2, 7)
    NIMBUS_CASE(3, 7)
    NIMBUS_CASE(4, 7)
    NIMBUS_CASE(2, 8)
    NIMBUS_CASE(3, 8)
    NIMBUS_CASE(4, 8)
#undef NIMBUS_CASE
    return hipErrorInvalidValue;
}

}  // namespace nimbus
