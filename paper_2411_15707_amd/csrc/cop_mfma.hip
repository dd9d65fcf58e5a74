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
// diagonal, so |D_d| <= k * min(DX,DQ) * 2^14, which the host keeps below 2^31.
// The epilogue rebuilds the 128-bit signed sum, adds a multiple of q that makes
// it non-negative, OFFX*S and the mask, and reduces once.
//
// Operand tiles are 32 x 32 bytes stored in the register order of the MFMA: the
// 16 bytes of lane l belong to row (or column) l % 32 and to k-slots
// (l / 32) * 16 .. +15 of the tile.  The A and B operands of the instruction
// use the same lane/byte -> k mapping, so any fixed assignment of k-slots to
// actual k indices gives the same sum as long as both sides share it.
#include "cop_common.hpp"

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
    LimbTable limbs;
    uint64_t bias_hi[kMaxLimbs], bias_lo[kMaxLimbs];   // q_l << sh
};

constexpr int KS = 4;         // k-blocks (of 32) per LDS stage

template <int DX, int DQ>
__global__ __launch_bounds__(256) void cop_mfma_kernel(const MfmaArgs a)
{
    constexpr int ND = DX + DQ - 1;
    constexpr int STAGE = KS * DQ * 64;             // uint4 per stage
    constexpr int PER_THREAD = STAGE / 256;         // = DQ for KS = 4
    static_assert(STAGE % 256 == 0, "stage must split evenly over the workgroup");
    __shared__ uint4 ldsB[2][STAGE];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

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

    const int KB = a.KB;
    const uint4 *gB = a.planes + (size_t)ct * KB * (DQ * 64);
    const uint4 *gA = a.xd + (size_t)rt * KB * (DX * 64) + lane;   // dereferenced only if active

    v16i acc[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[d][r] = 0;

    const int nstages = (KB + KS - 1) / KS;
    const int total_u4 = KB * DQ * 64;              // uint4 of B for this column tile

    // prologue: stage 0 -> LDS buffer 0
    {
#pragma unroll
        for (int u = 0; u < PER_THREAD; ++u) {
            const int idx = u * 256 + (int)threadIdx.x;
            if (idx < total_u4) ldsB[0][idx] = gB[idx];
        }
    }
    v4i a_nxt[DX];
    if (active) {
#pragma unroll
        for (int d = 0; d < DX; ++d) {
            const uint4 t = gA[d * 64];
            a_nxt[d] = (v4i){(int)t.x, (int)t.y, (int)t.z, (int)t.w};
        }
    }
    __syncthreads();

    for (int s = 0; s < nstages; ++s) {
        const int buf = s & 1;
        // global loads of the next stage, kept in registers until this stage is consumed
        uint4 stg[PER_THREAD];
        const int next_base = (s + 1) * STAGE;
#pragma unroll
        for (int u = 0; u < PER_THREAD; ++u) {
            const int idx = next_base + u * 256 + (int)threadIdx.x;
            if (idx < total_u4) stg[u] = gB[idx];
        }

        if (active) {
            const int kb_end = (s * KS + KS < KB) ? KS : (KB - s * KS);
            for (int kk = 0; kk < kb_end; ++kk) {
                v4i a_cur[DX];
#pragma unroll
                for (int d = 0; d < DX; ++d) a_cur[d] = a_nxt[d];
                const int kb_next = s * KS + kk + 1;
                if (kb_next < KB) {
#pragma unroll
                    for (int d = 0; d < DX; ++d) {
                        const uint4 t = gA[((size_t)kb_next * DX + d) * 64];
                        a_nxt[d] = (v4i){(int)t.x, (int)t.y, (int)t.z, (int)t.w};
                    }
                }
                v4i b[DQ];
#pragma unroll
                for (int d = 0; d < DQ; ++d) {
                    const uint4 t = ldsB[buf][(kk * DQ + d) * 64 + lane];
                    b[d] = (v4i){(int)t.x, (int)t.y, (int)t.z, (int)t.w};
                }
#pragma unroll
                for (int dq = 0; dq < DQ; ++dq)
#pragma unroll
                    for (int dx = 0; dx < DX; ++dx)
                        acc[dx + dq] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                            a_cur[dx], b[dq], acc[dx + dq], 0, 0, 0);
            }
        }

#pragma unroll
        for (int u = 0; u < PER_THREAD; ++u) {
            const int idx = next_base + u * 256 + (int)threadIdx.x;
            if (idx < total_u4) ldsB[buf ^ 1][idx - next_base] = stg[u];
        }
        __syncthreads();
    }

    if (!active) return;

    // ---- epilogue: rebuild, add q*2^sh + OFFX*S + mask, reduce, store ----
    const uint32_t col = ct * kTile + (uint32_t)(lane & 31);
    const uint32_t limb = (col / (uint32_t)a.N) % (uint32_t)a.L;
    const Limb P = a.limbs.limb[limb];
    uint64_t base_hi = a.bias_hi[limb], base_lo = a.bias_lo[limb];
    {
        const uint64_t S = a.colsum[col];
        add128(base_hi, base_lo, __umul64hi(S, (uint64_t)a.offx), S * (uint64_t)a.offx);
    }
    const int row0 = rt * kTile + 4 * (lane >> 5);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = row0 + 8 * (r >> 2) + (r & 3);
        if (row < a.m) {
            // W0 = sum_{d<4} D_d 2^(8d), W1 = sum_{4<=d<8} D_d 2^(8(d-4)), W2 = rest
            int64_t W[3] = {0, 0, 0};
#pragma unroll
            for (int d = 0; d < ND; ++d)
                W[d >> 2] += (int64_t)acc[d][r] * (int64_t)(1 << (8 * (d & 3)));
            uint64_t lo = (uint64_t)W[0];
            uint64_t hi = (uint64_t)(W[0] >> 63);
            add128(hi, lo, (uint64_t)(W[1] >> 32), (uint64_t)W[1] << 32);
            hi += (uint64_t)W[2];
            add128(hi, lo, base_hi, base_lo);
            const size_t idx = (size_t)row * a.C + col;
            if (a.mask) add128(hi, lo, 0, a.mask[idx]);
            a.out[idx] = barrett128(hi, lo, P);
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

bool mfma_supported(const Problem &p)
{
    const int DX = planes_x(p.x_bits), DQ = planes_q(p.q_bits_max);
    if (DX < 2 || DX > 4 || DQ < 7 || DQ > 8) return false;
    const long long pairs = DX < DQ ? DX : DQ;
    // zero padding of k adds nothing to |D_d|
    return (long long)p.k * pairs * 16384ll <= 2147483647ll;
}

template <int DQ>
static hipError_t prepare_impl(const Problem &p, const uint64_t *ctW, void *prepared,
                               hipStream_t stream)
{
    const int KB = (p.k + kTile - 1) / kTile;
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
    const int KB = (p.k + kTile - 1) / kTile;
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
    const int KB = (p.k + kTile - 1) / kTile;
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
    a.limbs = p.limbs;
    // q * 2^sh with 2^sh >= k * 2^(8 DX - 1) >= |sum x' c'| / q
    const int sh = ceil_log2((unsigned)p.k) + 8 * DX - 1;
    for (int l = 0; l < p.L; ++l) {
        const unsigned __int128 b = (unsigned __int128)p.limbs.limb[l].q << sh;
        a.bias_hi[l] = (uint64_t)(b >> 64);
        a.bias_lo[l] = (uint64_t)b;
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
