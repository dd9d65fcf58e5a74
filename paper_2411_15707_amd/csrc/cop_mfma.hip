// Matrix-core (int8 MFMA) kernels for the COP accumulation, gfx950.
//
// The contraction out = X * ctW (Algorithm 1 step 2 of the paper) is an exact
// integer matrix product with a 2^x_bits-bounded left operand and a q-bounded
// right operand.  Both are split into signed bytes so that the products run on
// v_mfma_i32_32x32x32_i8:
//
//   x  = x' + OFFX,  x' = sum_{a<DX} dx_a 256^a,  dx_a = byte_a(x) - 128 for the bytes that
//                    can reach 128 (8a + 8 <= x_bits), dx_a = byte_a(x) for the others (the
//                    top byte of a 20-bit share is a digit in [0, 15]: small operands keep
//                    the multipliers quieter, and the kernel's speed is set by power);
//                    OFFX = sum of 128 * 256^a over the shifted bytes   (no carries needed)
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
// The epilogue forms V = sum_d D_d 256^d + (q << sh) + OFFX*S + mask, where the
// multiple of q makes the total non-negative, and reduces V once.
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
    const uint64_t *__restrict__ X, int m, int k, int KB, uint32_t total, uint32_t offx,
    int half_shift, uint32_t *__restrict__ xd)
{
    // one thread = four consecutive k of one row: one 32-bit word in each of the DX planes
    const uint32_t gid = blockIdx.x * 256u + threadIdx.x;
    if (gid >= total) return;
    const uint32_t word = gid & 3u;                 // which 4 of the lane's 16 k-slots
    const uint32_t lane = (gid >> 2) & 63u;
    const uint32_t tile = gid >> 8;                 // rt * KB + kb
    const uint32_t kb = tile % (uint32_t)KB;
    const uint32_t rt = tile / (uint32_t)KB;
    const int row = (int)rt * kTile + (int)(lane & 31u);
    const int kbase = (int)kb * kTile + (int)(lane >> 5) * 16 + (int)word * 4;

    uint32_t w[DX];
#pragma unroll
    for (int d = 0; d < DX; ++d) w[d] = 0;
    if (row < m) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int i = kbase + b;
            if (i < k) {
                // flipping bit 7 of a byte turns it into the two's complement digit byte - 128
                // (half_shift = 32 selects the upper half of a share wider than 32 bits)
                const uint32_t x = (uint32_t)(X[(size_t)row * k + i] >> half_shift) ^ offx;
#pragma unroll
                for (int d = 0; d < DX; ++d) w[d] |= ((x >> (8 * d)) & 0xffu) << (8 * b);
            }
        }
    }
#pragma unroll
    for (int d = 0; d < DX; ++d)
        xd[(((size_t)tile * DX + d) * 64u + lane) * 4u + word] = w[d];
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
    uint32_t kb_magic;        // floor(2^32 / KB): x / KB = umulhi(x, kb_magic) or one more
    uint32_t log_n;           // N = 2^log_n
    uint32_t l_magic;         // ceil(2^32 / L) for L >= 2: x / L = umulhi(x, l_magic) for x < 2^31
    uint32_t offx;            // OFFX
    uint64_t q[kMaxLimbs];
    double qinv[kMaxLimbs];   // 1 / q_l, rounded
    // q_l << sh
    uint64_t cst_hi[kMaxLimbs], cst_lo[kMaxLimbs];
};

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
// Every tile carries the streaming hint: the ciphertext planes are read once and should not
// push the X planes out of L2, and for the X planes, which all workgroups of an XCD read
// within a few microseconds of each other, the hint makes no measurable difference; one kind
// of load lets all eight waves run the same instructions.
__device__ __forceinline__ void dma_tile(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_off,
                                         uint32_t uniform_off, void *dst_wave)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (NIMBUS_AS3 void *)dst_wave, 16, lane_off,
                                             uniform_off, 0, 2);
}

// The pipeline.  A workgroup of eight waves (two per SIMD) owns 128 token rows x 64
// coefficient columns; wave (wr, wc) owns the 32 x 32 output tile of row tile wr and
// column tile wc, with DX+DQ-1 int32 accumulator tiles.
//
// A stage is one k-block (32 values of k): 4*DX operand tiles of X (12 KB for DX = 3)
// and 2*DQ operand tiles of ciphertext planes (14 KB for DQ = 7), each in an LDS ring of
// its own.  Both are filled by direct-to-LDS loads of whole tiles (64 lanes x 16 B; the
// texture address unit spends the same time on narrower loads); nothing passes through
// registers on the way in.  The X tiles of a stage are dealt to waves 0-3, the ciphertext
// tiles to waves 4-7 (one wave of each kind per SIMD).  A wave knows how many loads it
// issues per stage, so "stage s has landed" is a wait on the number of its younger loads,
// then the barrier.
//
// Inside a wave the loop is software pipelined: the LDS reads of stage s+1 are issued
// between the matrix-core instructions of stage s, into the other of two operand sets.
//
// What the loop is bound by (measured).  Its duration follows the operand values: the
// chip lowers its clock under the combined matrix-core and memory load, and a k-block
// costs the matrix-core time of its 42 instructions per SIMD at the rate a register-only
// loop reaches on random bytes, plus a memory-side term; the two add up instead of
// overlapping.  Within that, what the schedule has to respect: enough bytes in flight per
// CU (a streaming read reaches 3.9 TB/s chip-wide with 8 KB in flight per CU, 6.5 with 16 KB,
// 7.0 from 32 KB on, direct-to-LDS and register loads alike; two to three stages of 26 KB
// are in flight here), the ciphertext loads spread over the iteration, where the other
// wave of the SIMD can fill a gap with its own matrix-core instructions, and
// instruction issue (a wave issues an instruction every four or five
// cycles at best and all eight waves run in lockstep between barriers, so every scalar
// instruction costs: one stage issued per iteration from the first iteration on,
// ring offsets carried and wrapped instead of recomputed, and the wait for "at most n
// loads pending", an immediate of the instruction, done by a computed jump).

template <int DX, int DQ>
struct Pipe {
    static constexpr int ND = DX + DQ - 1;
    static constexpr int A_TILES = 4 * DX;
    static constexpr int B_TILES = 2 * DQ;
    static constexpr int A_BYTES = A_TILES * kTileBytes;
    static constexpr int B_BYTES = B_TILES * kTileBytes;
    // accumulators + two operand sets + addressing must fit 256 registers (two waves per SIMD)
    static constexpr bool PIPELINED = ND * 16 + 2 * (DX + DQ) * 4 + 12 <= 256;
    static constexpr int AHEAD = PIPELINED ? 1 : 0;
    // Lead: stages 0 .. LEAD-1 are issued up front, iteration s issues stage s + LEAD
    // after its barrier, into the slot of stage s + LEAD - RING.  That slot has been read
    // by every wave once all have passed the barrier of iteration s + LEAD - RING + 1 -
    // AHEAD, so RING = LEAD + 1 - AHEAD slots are enough.
    static constexpr int LEAD = 3;
    static constexpr int RING = LEAD + 1 - AHEAD;
    static_assert(LEAD >= 1 + AHEAD, "the stage read next must have been issued");
    // X tile t goes to wave t % 4 as its load t / 4, ciphertext tile t to wave 4 + t % 4
    static constexpr int MAXU = ((A_TILES > B_TILES ? A_TILES : B_TILES) + 3) / 4;
    static_assert((LEAD - 1) * MAXU <= 63, "pending-load count must fit the wait counter");
    static constexpr int LDS_BYTES = RING * (A_BYTES + B_BYTES);
    static_assert(LDS_BYTES <= 160 * 1024, "rings do not fit the LDS");
};

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

// FULL: m is a multiple of 128, so every wave has its 32 rows: the code for waves without
// rows and the row tests around the loads and stores of the epilogue (a compare, an exec
// update and a branch each) are left out.
//
// MASKLDS: the workgroup's 128 x 64 mask words (64 KB) are brought into LDS by the first
// iterations of the loop, one direct-to-LDS load per wave and iteration, instead of being
// read from memory when the loop is over: the 16 B per output that mask and result move
// would otherwise all fall into the last microseconds of the launch, where they are the
// only traffic and every workgroup asks at once.  Needs a mask, m a multiple of 128, a
// pipelined variant, room in the LDS, at least kMaskLdsMinKB k-blocks and a row block whose
// mask rows span less than 4 GB (host: mask_in_lds()).
constexpr int kMaskTileBytes = 128 * 64 * 8;
constexpr int kMaskLoads = kMaskTileBytes / kTileBytes / 8;     // per wave: 8
constexpr int kMaskPhase = kMaskLoads + 2;                      // iterations that count them

template <int DX, int DQ, bool FULL, bool MASKLDS>
__global__ __launch_bounds__(512, 1) void cop_mfma_kernel(const MfmaArgs a)
{
    using P_ = Pipe<DX, DQ>;
    // Every scalar argument the setup needs, asked for in one batch: left to the compiler the
    // loads sit next to their first uses, and the setup waits for the constant cache once
    // per group of them instead of once.
    asm volatile("" ::"s"(a.xd), "s"(a.planes), "s"(a.colsum), "s"(a.m), "s"(a.KB), "s"(a.RB),
                 "s"(a.L), "s"(a.CT), "s"(a.kb_magic), "s"(a.log_n), "s"(a.l_magic));
    constexpr int ND = P_::ND;
    constexpr bool PIPELINED = P_::PIPELINED;
    constexpr int AHEAD = P_::AHEAD, LEAD = P_::LEAD, RING = P_::RING;
    constexpr int SETS = PIPELINED ? 2 : 1;
    static_assert(!MASKLDS || (FULL && P_::PIPELINED && P_::LDS_BYTES + kMaskTileBytes <= 160 * 1024),
                  "mask tile in LDS: full row blocks, pipelined variant, and it must fit");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[P_::LDS_BYTES + (MASKLDS ? kMaskTileBytes : 0)];
    unsigned char *const ldsA = lds;
    unsigned char *const ldsB = lds + RING * P_::A_BYTES;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // 0..7
    const int wr = wave >> 1, wc = wave & 1;

    // workgroup -> (64-column tile, row block).  Workgroups are dealt round-robin to
    // the 8 XCDs; the RB row blocks that share a column tile are kept on one XCD
    // and adjacent in launch order so that tile is fetched from HBM once.
    uint32_t ct2, rb;
    {
        const uint32_t id = blockIdx.x;
        const uint32_t CT2 = a.CT >> 1;
        if (a.RB == 1) {                            // one row block: no division
            rb = 0;
            ct2 = id;
        } else if ((CT2 & 7u) == 0) {
            const uint32_t xcd = id & 7u, slot = id >> 3;
            rb = slot % (uint32_t)a.RB;
            ct2 = (slot / (uint32_t)a.RB) * 8u + xcd;
        } else {
            rb = id % (uint32_t)a.RB;
            ct2 = id / (uint32_t)a.RB;
        }
    }
    const int RT = (a.m + kTile - 1) / kTile;       // row tiles that exist in the workspace
    const int rt = (int)rb * 4 + wr;                // this wave's row tile
    const bool active = FULL || rt < RT;            // wave-uniform
    const int KB = a.KB;

    // ---- this wave's share of the loads of one stage (sources at k-block 0) ----
    // Waves 0-3 (the first wave of each SIMD) load the X tiles, from L2: wave w the DX planes
    // of row tile w of the row block (clamped to a row tile that exists; rows past m are
    // never used).  Waves 4-7 (the second of each SIMD) load the ciphertext tiles, from HBM:
    // waves 4 and 5 the planes of the first column tile (planes 0-3 and 4 .. DQ-1), waves 6
    // and 7 those of the second.  A load's source is the wave's buffer descriptor (base of
    // the workgroup's X or ciphertext region), the lane's 16 bytes, and a wave-uniform
    // offset: the tile's place at k-block 0 plus the carried k-block offset.  (A row tile or
    // column tile of planes spans KB * D KiB < 2^23 bytes.  Everything up to the first loads
    // is scalar work on the critical path of the launch: no divisions, and whatever the loads
    // do not need comes after them.)
    const uint32_t a_tile_bytes = (uint32_t)KB * DX * kTileBytes;     // one row tile, all k-blocks
    const uint32_t b_tile_bytes = (uint32_t)KB * DQ * kTileBytes;     // one column tile
    const unsigned char *const a_base =
        (const unsigned char *)a.xd + (size_t)rb * 4u * a_tile_bytes;
    const unsigned char *const b_base =
        (const unsigned char *)a.planes + (size_t)ct2 * 2u * b_tile_bytes;
    const bool loads_x = wave < 4;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(loads_x ? a_base : b_base), 0, 0xffffffff, 0x00027000);
    const uint32_t lane16 = (uint32_t)lane * 16u;
    constexpr int PH = (DQ + 1) / 2;                // planes of a column tile on its first wave
    static_assert(P_::MAXU == 4 && DX <= 4 && PH <= 4, "four load slots per wave and stage");
    uint32_t toff[P_::MAXU];                        // the tile's byte offset at k-block 0
    uint32_t dst[P_::MAXU];                         // the tile's byte offset in slot 0 of the LDS
    int n_loads;                                    // loads per stage
    {
        uint32_t first_off, first_tile;             // of the wave's first tile; the others follow it
        if (loads_x) {
            int r = wave;
            const int last = RT - 1 - (int)rb * 4;  // last row tile of the block that exists (>= 0)
            if (r > last) r = last;
            first_off = (uint32_t)r * a_tile_bytes;
            first_tile = (uint32_t)wave * DX;
            n_loads = DX;
        } else {
            const uint32_t c = (uint32_t)(wave >> 1) & 1u, hi = (uint32_t)wave & 1u;
            first_off = c * b_tile_bytes + hi * (PH * kTileBytes);
            first_tile = (uint32_t)P_::A_TILES * RING + c * DQ + hi * PH;
            n_loads = hi ? DQ - PH : PH;
        }
#pragma unroll
        for (int u = 0; u < P_::MAXU; ++u) {
            toff[u] = first_off + (uint32_t)u * kTileBytes;
            dst[u] = (first_tile + (uint32_t)u) * kTileBytes;
        }
    }
    // Stage s of this workgroup is k-block (s + k_start) mod KB: the sum over k does not
    // care about the order, and workgroups that walk their (equally spaced) ciphertext
    // regions in lockstep would otherwise ask the same memory channels for data at the
    // same moment.
    uint32_t k_start = blockIdx.x - __umulhi(blockIdx.x, a.kb_magic) * (uint32_t)KB;   // id mod KB
    if (k_start >= (uint32_t)KB) k_start -= (uint32_t)KB;
    // Wave-uniform state of the issue side, for the next stage to issue: byte offset of
    // its k-block in the source, byte offset of its slot in the ring.  Carried and
    // wrapped, never recomputed.
    const uint32_t src_step = (uint32_t)(loads_x ? DX : DQ) * kTileBytes;   // per k-block
    const uint32_t src_end = (uint32_t)KB * src_step;
    const uint32_t slot_step = loads_x ? P_::A_BYTES : P_::B_BYTES;
    const uint32_t slot_end = RING * slot_step;
    uint32_t src_off = k_start * src_step;
    uint32_t slot_off = 0;
    auto bump = [](uint32_t v, uint32_t step, uint32_t end) -> uint32_t {
        v += step;
        return v == end ? 0u : v;
    };
    // load u of the stage at the carried offsets
    auto issue_one = [&](auto u_c) {
        constexpr int u = decltype(u_c)::value;
        unsigned char *const d = lds + (dst[u] + slot_off);
        dma_tile(rsrc, lane16, toff[u] + src_off, d);
    };
#define NIMBUS_NEXT_ISSUE()                                                   \
    do {                                                                      \
        src_off = bump(src_off, src_step, src_end);                           \
        slot_off = bump(slot_off, slot_step, slot_end);                       \
    } while (0)

    // ---- up front: stages 0 .. LEAD-1 ----
    // The accumulators are cleared between the stages: the memory pipeline takes the first
    // loads of a launch slowly (nothing is translated or cached yet), and the moves fill
    // the time the wave would spend waiting for it to accept the next one.
    v16i acc[ND];
#pragma unroll
    for (int st = 0; st < LEAD; ++st) {
        if (st < KB) {
            static_for<0, P_::MAXU>([&](auto u_c) {
                if (decltype(u_c)::value < n_loads) issue_one(u_c);
            });
            NIMBUS_NEXT_ISSUE();
        }
#pragma unroll
        for (int d = st; d < ND; d += LEAD) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[d][r] = 0;
            tie_acc(acc[d]);
        }
    }

    // ---- what the first loads did not need ----
    __builtin_amdgcn_sched_barrier(0);
    n_loads = __builtin_amdgcn_readfirstlane(n_loads);
    // The column's ciphertext sum is needed after the loop; asked for now it costs two
    // registers, not a round trip to memory at the end.  An ordinary load: the compiler places
    // the wait for it at its first use, and the statements below that clobber memory keep the
    // load itself up here.  (One more load ahead of the loop's counted waits only makes them
    // wait for it too; it is the oldest but LEAD stages by then.)
    const uint64_t colsum_S =
        a.colsum[(ct2 * 2u + (uint32_t)wc) * kTile + (uint32_t)(lane & 31)];
    asm volatile("" ::: "memory");
    // The limb of this wave's 32 columns (they lie in one (polynomial, limb) block of N >= 32
    // columns), worked out here with a shift and a multiply-high: after the loop it would sit
    // on the path to the first loads of the epilogue.
    uint32_t limb;
    {
        const uint32_t blk = ((ct2 * 2u + (uint32_t)wc) * kTile) >> a.log_n;
        limb = a.L == 1 ? 0u : blk - (uint32_t)a.L * __umulhi(blk, a.l_magic);
        limb = __builtin_amdgcn_readfirstlane(limb);
        asm volatile("" : "+s"(limb));
    }

    // Operands come out of LDS through explicit ds_read_b128 instructions: reads the
    // compiler can see would each be made to wait for every direct-to-LDS load in flight.
    const uint32_t lds0 = (uint32_t)(uintptr_t)(NIMBUS_AS3 void *)&lds[0];
    const uint32_t laneA = lds0 + (uint32_t)(wr * DX) * kTileBytes + (uint32_t)lane * 16u;
    const uint32_t laneB = lds0 + (uint32_t)(RING * P_::A_BYTES) +
                           (uint32_t)(wc * DQ) * kTileBytes + (uint32_t)lane * 16u;
    // ring offsets of the stage that is read next
    uint32_t rdA = 0, rdB = 0;
#define NIMBUS_NEXT_READ()                                                    \
    do {                                                                      \
        rdA = bump(rdA, P_::A_BYTES, RING * P_::A_BYTES);                     \
        rdB = bump(rdB, P_::B_BYTES, RING * P_::B_BYTES);                     \
    } while (0)
    v4i xa[SETS][DX], xb[SETS][DQ];                 // [operand set][plane]
    // read number i (0 <= i < DX+DQ) of the stage at (rdA, rdB) into operand set SET
    auto read_one = [&](auto set_c, auto i_c) {
        constexpr int SET = decltype(set_c)::value;
        constexpr int i = decltype(i_c)::value;
        if constexpr (i < DX)
            xa[SET][i] = lds_read_b128<i * kTileBytes>(laneA + rdA);
        else
            xb[SET][i - DX] = lds_read_b128<(i - DX) * kTileBytes>(laneB + rdB);
    };
    auto read_ops = [&](auto set_c) {
        static_for<0, DX + DQ>([&](auto i_c) { read_one(set_c, i_c); });
    };
    // all LDS reads of this wave are back; ties every register of the set to the wait
    auto wait_ops = [&](auto set_c) {
        constexpr int SET = decltype(set_c)::value;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int d = 0; d < DX; ++d) tie(xa[SET][d]);
#pragma unroll
        for (int d = 0; d < DQ; ++d) tie(xb[SET][d]);
    };

    // Loads of this wave younger than those of stage j = s + AHEAD, before iteration s:
    // stages j+1 .. min(KB, s + LEAD) - 1, that is min(LEAD - 1 - AHEAD, KB - 1 - j) stages.
    // No stage j: nothing to wait for.
    auto younger = [&](int s) -> int {
        const int j = s + AHEAD;
        if (j >= KB) return 63;
        int st = KB - 1 - j;
        if (st > LEAD - 1 - AHEAD) st = LEAD - 1 - AHEAD;
        return st * n_loads;
    };
    asm volatile("" ::: "memory");
    if constexpr (PIPELINED) {
        // stage 0 is read before the loop; its younger loads are those of stages 1 .. LEAD-1
        const int st = (KB < LEAD ? KB : LEAD) - 1;
        wait_vmem_n(st * n_loads);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (active) read_ops(std::integral_constant<int, 0>{});
        NIMBUS_NEXT_READ();
    }

    // iteration s, pipelined: make stage s+1 visible, issue stage s+LEAD into a slot
    // whose stage every wave has in registers, read stage s+1 into the other operand
    // set, run the matrix cores on stage s.  Not pipelined (register budget of the
    // widest variants): make stage s visible, issue, read stage s, wait, run.
    //
    // Between consecutive matrix-core instructions goes at most one other instruction
    // (all eight waves leave the barrier together: a burst of loads or LDS reads would
    // fill the queues of the CU and hold back the matrix-core instructions behind it):
    // first the X loads, then the LDS reads of stage s+1 (pipelined variants), the
    // ciphertext loads last.  The empty volatile asm statements pin this order.
    constexpr int R0 = PIPELINED ? DX + DQ : 0;     // LDS reads placed between the MFMAs
    constexpr int NPOS = DX * DQ;
    static_assert(NPOS >= R0 + 1 && NPOS >= P_::MAXU, "not enough positions between the MFMAs");
    // positions: [0, MAXU) X loads, [RP0, RP0 + R0) reads, the last MAXU ciphertext loads
    constexpr int RP0 = P_::MAXU < NPOS - R0 ? P_::MAXU : NPOS - R0;
    constexpr int XP0 = NPOS - P_::MAXU;
    // ACTIVE: the wave has rows.
    auto iteration = [&](int s, auto set_c, auto active_c) {
        constexpr int SET = decltype(set_c)::value;
        constexpr bool ACTIVE = decltype(active_c)::value;
        wait_vmem_n(younger(s));
        if constexpr (PIPELINED && ACTIVE) wait_ops(set_c);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if constexpr (!PIPELINED && ACTIVE) {
            read_ops(set_c);
            wait_ops(set_c);
        }
        const int issue_n = s + LEAD < KB ? n_loads : 0;    // stage s + LEAD exists: its loads
        static_for<0, NPOS>([&](auto i_c) {
            constexpr int i = decltype(i_c)::value;
            constexpr int dx = i / DQ, dq = i % DQ;
            if constexpr (ACTIVE) {
                tie(xa[SET][dx]);
                tie(xb[SET][dq]);
                acc[dx + dq] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                    xa[SET][dx], xb[SET][dq], acc[dx + dq], 0, 0, 0);
                tie_acc(acc[dx + dq]);
            }
            if constexpr (i < P_::MAXU) {
                if (loads_x && i < issue_n) issue_one(i_c);
            }
            if constexpr (i >= RP0 && i < RP0 + R0) {
                // (the last iteration reads a stale slot: valid LDS, never used)
                if constexpr (ACTIVE)
                    read_one(std::integral_constant<int, (PIPELINED ? 1 - SET : SET)>{},
                             std::integral_constant<int, i - RP0>{});
            }
            if constexpr (i >= XP0) {
                constexpr int u = i - XP0;
                if (!loads_x && u < issue_n) issue_one(std::integral_constant<int, u>{});
            }
        });
        asm volatile("" ::: "memory");
    };
    // Steady state, pipelined variants: as long as stage s + LEAD exists every load of the
    // iteration is issued and the number of younger loads is the same every time.  All
    // waves run the same instructions: the first NMIN loads of a stage are unconditional
    // (every wave has that many), the others hang on one scalar test each.
    constexpr int NMIN = DX < P_::B_TILES / 4 ? DX : P_::B_TILES / 4;
    // The barrier of an iteration does not stand in front of its first matrix-core
    // instructions: their operands are in registers already.  What has to follow it are the
    // LDS reads of the next stage (its loads have landed everywhere) and the loads into the
    // slot of the stage that every wave now holds in registers (each passed its LDS wait at
    // the top).  With the barrier after instruction NPRE - 1, the wave of a SIMD that arrives
    // first has left work in the matrix-core queue, and the later one finds the pipe free for
    // its own first instructions: the pipe does not drain while the waves synchronise.
    constexpr int NPRE = 4 < NPOS / 3 ? 4 : NPOS / 3;
    // behind the barrier: the loads, then the reads, spread evenly over the remaining positions
    constexpr int NITEMS = P_::MAXU + R0, SPAN = NPOS - NPRE;
    // Mask tile (MASKLDS): load j of the tile, 0 <= j < 64, brings rows 2j and 2j+1 of the
    // row block (lanes 0-31 and 32-63, 16 bytes = two columns each) to LDS bytes
    // [j KB, j KB + 1 KB) of the tile, which so ends up row-major [128][64].  Wave w issues
    // load w + 8 i in iteration i < kMaskLoads, ahead of the iteration's stage loads; a
    // wait for a stage then has one more younger load to allow for in iterations
    // 1 .. kMaskLoads.  Rows past the end of the mask (none, m being a multiple of 128) would
    // read as zero: the descriptor ends where the mask ends.
    __amdgpu_buffer_rsrc_t rsrc_m = rsrc;
    uint32_t voff_m = 0, soff_m = 0, dst_m = 0;
    if constexpr (MASKLDS) {
        const uint64_t first = ((uint64_t)rb * 128u * a.C + (uint64_t)ct2 * 64u) * 8u;
        const uint64_t left = (uint64_t)a.m * a.C * 8u - first;
        rsrc_m = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((const unsigned char *)a.mask + first), 0,
            left > 0xffffffffull ? 0xffffffffu : (uint32_t)left, 0x00027000);
        voff_m = (uint32_t)(lane >> 5) * a.C * 8u + (uint32_t)(lane & 31) * 16u;
        soff_m = (uint32_t)wave * 2u * a.C * 8u;
        dst_m = (uint32_t)P_::LDS_BYTES + (uint32_t)wave * kTileBytes;
    }
    auto steady_iteration = [&](auto set_c, auto phase_c, int t) {
        constexpr int SET = decltype(set_c)::value;
        constexpr bool MASKPHASE = decltype(phase_c)::value;   // iteration t < kMaskPhase
        constexpr int W = LEAD - 1 - AHEAD;
        wait_ops(set_c);
        static_for<0, NPOS>([&](auto i_c) {
            constexpr int i = decltype(i_c)::value;
            constexpr int dx = i / DQ, dq = i % DQ;
            tie(xa[SET][dx]);
            tie(xb[SET][dq]);
            acc[dx + dq] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                xa[SET][dx], xb[SET][dq], acc[dx + dq], 0, 0, 0);
            tie_acc(acc[dx + dq]);
            if constexpr (i == NPRE - 1) {
                if constexpr (MASKPHASE)
                    wait_vmem_n(W * n_loads + ((t >= 1 && t <= kMaskLoads) ? 1 : 0));
                else
                    wait_vmem_loads<W, P_::MAXU, NMIN>(n_loads);
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if constexpr (MASKPHASE) {
                    if (t < kMaskLoads) {
                        dma_tile(rsrc_m, voff_m, soff_m, lds + dst_m);
                        soff_m += 16u * a.C * 8u;
                        dst_m += 8u * kTileBytes;
                    }
                }
            }
            if constexpr (i >= NPRE) {
                static_for<0, NITEMS>([&](auto j_c) {
                    constexpr int j = decltype(j_c)::value;
                    if constexpr (NPRE + j * SPAN / NITEMS == i) {
                        if constexpr (j < P_::MAXU) {
                            if (j < NMIN || j < n_loads)
                                dma_tile(rsrc, lane16, toff[j] + src_off,
                                                lds + (dst[j] + slot_off));
                        } else {
                            read_one(std::integral_constant<int, 1 - SET>{},
                                     std::integral_constant<int, j - P_::MAXU>{});
                        }
                    }
                });
            }
        });
        asm volatile("" ::: "memory");
    };
    // the carried offsets move on between iterations (outside the lambda: plain locals)
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    if (!active) {
        for (int s = 0; s < KB; ++s) {
            iteration(s, C0{}, std::false_type{});
            NIMBUS_NEXT_ISSUE();
        }
        return;
    }
    if constexpr (PIPELINED) {
        int s = 0;
        if constexpr (MASKLDS) {
            static_assert(kMaskPhase % 2 == 0, "whole pairs of iterations");
            for (; s < kMaskPhase; s += 2) {        // the host made sure KB - LEAD >= kMaskPhase
                steady_iteration(C0{}, std::true_type{}, s);
                NIMBUS_NEXT_ISSUE();
                NIMBUS_NEXT_READ();
                steady_iteration(C1{}, std::true_type{}, s + 1);
                NIMBUS_NEXT_ISSUE();
                NIMBUS_NEXT_READ();
            }
        }
        for (; s + 2 <= KB - LEAD; s += 2) {        // iterations below KB - LEAD are steady
            steady_iteration(C0{}, std::false_type{}, s);
            NIMBUS_NEXT_ISSUE();
            NIMBUS_NEXT_READ();
            steady_iteration(C1{}, std::false_type{}, s + 1);
            NIMBUS_NEXT_ISSUE();
            NIMBUS_NEXT_READ();
        }
        for (; s < KB; s += 2) {
            iteration(s, C0{}, std::true_type{});
            NIMBUS_NEXT_ISSUE();
            NIMBUS_NEXT_READ();
            if (s + 1 < KB) {
                iteration(s + 1, C1{}, std::true_type{});
                NIMBUS_NEXT_ISSUE();
                NIMBUS_NEXT_READ();
            }
        }
    } else {
        for (int s = 0; s < KB; ++s) {
            iteration(s, C0{}, std::true_type{});
            NIMBUS_NEXT_ISSUE();
            NIMBUS_NEXT_READ();
        }
    }
#undef NIMBUS_NEXT_ISSUE
#undef NIMBUS_NEXT_READ
    // the last pipelined iteration has read a stage that does not exist into the other
    // operand set; nothing may reuse those registers before the reads are back
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

    // ---- epilogue: rebuild, add the constant and the mask, reduce, store ----
    const uint32_t col = (ct2 * 2u + (uint32_t)wc) * kTile + (uint32_t)(lane & 31);
    const uint64_t q = a.q[limb];
    const double qinv = a.qinv[limb];
    const int row0 = rt * kTile + 4 * (lane >> 5);
    // every load of the epilogue first (mask words, then the column sum), so that their
    // latencies overlap
    // element r of the lane is row row0 + roff(r); addresses are the lane's address of
    // row0 plus a wave-uniform multiple of the row length
    auto roff = [](int r) -> int { return 8 * (r >> 2) + (r & 3); };
    const size_t lane_elem = (size_t)row0 * a.C + col;
    const uint64_t *const mask0 = a.mask ? a.mask + lane_elem : nullptr;
    const uint64_t *const prev0 = a.prev ? a.prev + lane_elem : nullptr;
    uint64_t *const out0 = a.out + lane_elem;
    uint64_t mk[16];                                // read once: streaming loads
    if constexpr (MASKLDS) {
        // the tile is in LDS, row-major [128][64]; every load of it landed before a barrier
        // of the loop that this wave has passed
        const unsigned char *const tile =
            lds + P_::LDS_BYTES + (uint32_t)(wr * kTile + 4 * (lane >> 5)) * 512u +
            (uint32_t)(wc * kTile + (lane & 31)) * 8u;
#pragma unroll
        for (int r = 0; r < 16; ++r) mk[r] = *(const uint64_t *)(tile + roff(r) * 512);
    } else if (a.mask) {
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
    if (a.prev) {
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
    double qinv_v = qinv, magic_c = 1688849860263936.0 - 0.5;      // 3 * 2^49 - 1/2
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
        // remainder modulo 2^64: lo - (qh 2^32 + ql) q, in [0, 2q); then one correction
        const uint64_t t = (((uint64_t)lo_hi << 32) | lo_lo) - (uint64_t)ql * q_lo;
        const uint32_t t_lo = (uint32_t)t;
        const uint32_t t_hi = (uint32_t)(t >> 32) - (ql * q_hi + qh * q_lo);   // upper word only
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

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static int ceil_log2(unsigned v)
{
    int b = 0;
    while ((1ull << b) < v) ++b;
    return b;
}

// OFFX: 128 in every byte of a share that can reach 128.  The same word is the XOR mask that
// turns those bytes into signed digits.
static uint32_t share_offset(int x_bits, int DX)
{
    uint32_t off = 0;
    for (int d = 0; d < DX; ++d)
        if (x_bits >= 8 * d + 8) off |= 0x80u << (8 * d);
    return off;
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
    // one workgroup per 128 x 64 output tile in a one-dimensional grid
    const uint64_t workgroups = (uint64_t)(p.C / (2 * kTile)) * (uint64_t)((p.m + 127) / 128);
    if (workgroups >= (1ull << 31)) return false;
    // the value reduced in the epilogue is below (2^(sh+1) + 2^33 + 1) * q (the second
    // 2^32 q: the previous pass of a wide share); the floating-point quotient needs it
    // below 2^47 * q
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
static hipError_t stage_impl(const Problem &p, const uint64_t *X, int half_shift, void *workspace,
                             hipStream_t stream)
{
    const int KB = kblocks(p.k);
    const int RT = (p.m + kTile - 1) / kTile;
    const uint32_t xtotal = (uint32_t)RT * KB * 256;
    hipLaunchKernelGGL(x_planes_kernel<DX>, dim3((xtotal + 255) / 256), dim3(256), 0, stream,
                       X, p.m, p.k, KB, xtotal, share_offset(p.x_bits, DX), half_shift,
                       (uint32_t *)workspace);
    return hipGetLastError();
}

// p.x_bits (<= 32) is the width of the half that is staged; half_shift is 0 or 32
hipError_t launch_stage_shares(const Problem &p, const uint64_t *X, int half_shift,
                               void *workspace, hipStream_t stream)
{
    switch (planes_x(p.x_bits)) {
    case 2: return stage_impl<2>(p, X, half_shift, workspace, stream);
    case 3: return stage_impl<3>(p, X, half_shift, workspace, stream);
    default: return stage_impl<4>(p, X, half_shift, workspace, stream);
    }
}

template <int DX, int DQ>
static hipError_t mfma_impl(const Problem &p, const void *staged, const void *prepared,
                            const uint64_t *mask, const uint64_t *prev, uint64_t *out,
                            hipStream_t stream)
{
    const int KB = kblocks(p.k);
    const uint32_t CT = (uint32_t)(p.C / kTile);

    MfmaArgs a{};
    a.xd = (const uint4 *)staged;
    a.planes = (const uint4 *)prepared;
    a.colsum = (const uint64_t *)((const char *)prepared + (size_t)CT * KB * DQ * kTileBytes);
    a.mask = mask;
    a.prev = prev;
    a.out = out;
    a.m = p.m;
    a.KB = KB;
    a.RB = (p.m + 127) / 128;
    a.N = p.N;
    a.L = p.L;
    a.C = (uint32_t)p.C;
    a.CT = CT;
    a.offx = share_offset(p.x_bits, DX);
    a.kb_magic = (uint32_t)((1ull << 32) / (uint64_t)KB);   // KB = 1: 2^32 does not fit, see below
    if (KB == 1) a.kb_magic = 0xffffffffu;
    a.log_n = 0;
    while ((1 << a.log_n) < p.N) ++a.log_n;
    a.l_magic = p.L >= 2 ? (uint32_t)(((1ull << 32) + (uint64_t)p.L - 1) / (uint64_t)p.L) : 0u;
    const int sh = bias_shift(p);
    for (int l = 0; l < p.L; ++l) {
        const uint64_t q = p.limbs.limb[l].q;
        const unsigned __int128 c = (unsigned __int128)q << sh;
        a.q[l] = q;
        a.qinv[l] = 1.0 / (double)q;
        a.cst_hi[l] = (uint64_t)(c >> 64);
        a.cst_lo[l] = (uint64_t)c;
    }
    const dim3 grid((CT / 2) * (uint32_t)a.RB);
    using P_ = Pipe<DX, DQ>;
    constexpr bool kCanMaskLds = P_::PIPELINED && P_::LDS_BYTES + kMaskTileBytes <= 160 * 1024;
    // mask tile in LDS: see the kernel; 128 rows of the mask must span less than 4 GB
    const bool mask_lds = kCanMaskLds && mask != nullptr && p.m % 128 == 0 &&
                          KB - P_::LEAD >= kMaskPhase && (uint64_t)p.C * 8u * 128u < (1ull << 32);
    if constexpr (kCanMaskLds) {
        if (mask_lds) {
            hipLaunchKernelGGL((cop_mfma_kernel<DX, DQ, true, true>), grid, dim3(512), 0, stream, a);
            return hipGetLastError();
        }
    }
    if (p.m % 128 == 0)
        hipLaunchKernelGGL((cop_mfma_kernel<DX, DQ, true, false>), grid, dim3(512), 0, stream, a);
    else
        hipLaunchKernelGGL((cop_mfma_kernel<DX, DQ, false, false>), grid, dim3(512), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_cop_mfma(const Problem &p, const void *staged, const void *prepared,
                           const uint64_t *mask, const uint64_t *prev, uint64_t *out,
                           hipStream_t stream)
{
    const int DX = planes_x(p.x_bits), DQ = planes_q(p.q_bits_max);
#define NIMBUS_CASE(dx, dq) \
    if (DX == dx && DQ == dq) return mfma_impl<dx, dq>(p, staged, prepared, mask, prev, out, stream);
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
