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
#include "cop_mfma_common.hpp"
#include <atomic>

namespace nimbus {

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
// (blockIdx.y: the problem, when the shares of several calls are staged in one launch)
struct StagePtrs {
    const uint64_t *X[kMaxBatch];
    uint32_t *xd[kMaxBatch];
};

template <int DX>
__global__ __launch_bounds__(256) void x_planes_kernel(
    const StagePtrs sp, int m, int k, int KB, uint32_t total, uint32_t offx, int half_shift)
{
    const uint64_t *__restrict__ const X = sp.X[blockIdx.y];
    uint32_t *__restrict__ const xd = sp.xd[blockIdx.y];
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

// The pipeline.  A workgroup of eight waves (two per SIMD) owns 128 token rows x 64
// coefficient columns; wave (wr, wc) owns the 32 x 32 output tile of row tile wr and
// column tile wc, with DX+DQ-1 int32 accumulator tiles.
//
// A stage is one k-block (32 values of k): 4*DX operand tiles of X (12 KB for DX = 3)
// and 2*DQ operand tiles of ciphertext planes (14 KB for DQ = 7), each in an LDS ring of
// its own.  Both are filled by direct-to-LDS loads of whole tiles (64 lanes x 16 B; the
// texture address unit spends the same time on narrower loads); nothing passes through
// registers on the way in.  Wave w < 4 loads the DX planes of row tile w, waves 4 and 5
// the two halves of the planes of the first column tile, waves 6 and 7 those of the
// second (one wave of each kind per SIMD, at most four loads per wave and stage).  A load
// is a buffer load: descriptor with the workgroup's base, the lane's 16 bytes, and one
// wave-uniform offset that is carried from stage to stage, so issuing it costs no vector
// arithmetic.  A wave knows how many loads it issues per stage, so "stage s has landed"
// is a wait on the number of its younger loads, then the barrier.
//
// Inside a wave the loop is software pipelined: the LDS reads of stage s+1 are issued
// between the matrix-core instructions of stage s, into the other of two operand sets.
// The steady state is one branch-free body that every wave runs: loads and reads sit at
// fixed places between the matrix-core instructions, the first few products of an
// iteration (whose operands were read during the iteration before) run in front of its
// barrier, and only the first and the last iterations are peeled.
//
// What the loop is bound by (measured).  Its duration follows the operand values: the
// chip lowers its clock under the combined matrix-core and memory load (1.5 to 1.8 GHz
// here against the 2.4 GHz of the data sheet), and a k-block costs the matrix-core time
// of its 42 instructions per SIMD, 1344 cycles, plus about a tenth.  Fewer cycles do
// not translate one to one: the chip answers a denser loop with a lower clock.  What the
// schedule has to respect: enough bytes in flight per CU (a streaming read reaches
// 3.9 TB/s chip-wide with 8 KB in flight per CU, 6.5 with 16 KB, 7.0 from 32 KB on,
// direct-to-LDS and register loads alike; three stages of 26 KB are in flight here), the
// ciphertext loads spread over the iteration, where the other wave of the SIMD can fill a
// gap with its own matrix-core instructions, and instruction issue (all eight waves run
// in lockstep between barriers, so every scalar instruction costs: ring offsets carried
// and wrapped instead of recomputed, and the wait for "at most n loads pending", an
// immediate of the instruction, done by a compare chain over the two or three counts
// that can occur).

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
    // load slots per wave and stage: a row tile's DX planes, or half of a column tile's DQ
    static constexpr int MAXU = ((A_TILES > B_TILES ? A_TILES : B_TILES) + 3) / 4;
    static_assert((LEAD - 1) * MAXU <= 63, "pending-load count must fit the wait counter");
    static constexpr int LDS_BYTES = RING * (A_BYTES + B_BYTES);
    static_assert(LDS_BYTES <= 160 * 1024, "rings do not fit the LDS");
};

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
//
// SHARED: the launch has several row blocks per column tile (m > 128).  They run on one XCD
// at the same time, start at the same k-block and load without the streaming hint, so the
// ciphertext tile comes over the fabric once and the other row blocks find it in the L2.
constexpr int kMaskTileBytes = 128 * 64 * 8;
constexpr int kMaskLoads = kMaskTileBytes / kTileBytes / 8;     // per wave: 8
constexpr int kMaskPhase = kMaskLoads + 2;                      // iterations that count them

template <int DX, int DQ, bool FULL, bool MASKLDS, bool SHARED>
__global__ __launch_bounds__(512, 1) void cop_mfma_kernel(const MfmaArgs a, const BatchPtrs b)
{
    using P_ = Pipe<DX, DQ>;
    // Every scalar argument the setup needs, asked for in one batch: left to the compiler the
    // loads sit next to their first uses, and the setup waits for the constant cache once
    // per group of them instead of once.
    asm volatile("" ::"s"(b.prob[0].xd), "s"(b.prob[0].planes), "s"(b.prob[0].colsum),
                 "s"(b.prob[0].mask), "s"(b.prob[0].out), "s"(b.count), "s"(a.m), "s"(a.KB), "s"(a.RB),
                 "s"(a.L), "s"(a.CT), "s"(a.kb_magic), "s"(a.log_n), "s"(a.l_magic));
    constexpr int ND = P_::ND;
    constexpr bool PIPELINED = P_::PIPELINED;
    constexpr int AHEAD = P_::AHEAD, LEAD = P_::LEAD, RING = P_::RING;
    constexpr int SETS = PIPELINED ? 2 : 1;
    static_assert(!MASKLDS || (FULL && P_::PIPELINED && P_::LDS_BYTES + kMaskTileBytes <= 160 * 1024),
                  "mask tile in LDS: full row blocks, pipelined variant, and it must fit");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[P_::LDS_BYTES + (MASKLDS ? kMaskTileBytes : 0)];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // 0..7
    const int wr = wave >> 1, wc = wave & 1;

    // tile id -> (64-column tile, row block).  A workgroup takes the tiles blockIdx.x,
    // blockIdx.x + gridDim.x, ... (the host launches one workgroup per compute unit when there
    // are more tiles than that).  Workgroups are dealt round-robin to the 8 XCDs, and with a
    // grid that is a multiple of 8 so are the tile ids; the RB row blocks that share a column
    // tile are kept on one XCD and adjacent in that order so that tile is fetched from HBM
    // once.  (The column tiles past the last multiple of 8, if any, are not worth the trouble.)
    // (the pointers of a single call are asked for with the first batch of scalar loads: an
    // indexed load would sit on the path to the first loads of the launch)
    const bool single = b.count == 1;
    // (a launch may hold several problems of the same shape: tile ids run through the first
    // problem's tiles, then the second's, ...; p is the problem)
    auto map_tile = [&](uint32_t id, uint32_t &p, uint32_t &ct2, uint32_t &rb) {
        p = 0;
        if (!single) {
            while (id >= b.tiles_each) {            // at most kMaxBatch - 1 rounds, scalar
                id -= b.tiles_each;
                ++p;
            }
        }
        const uint32_t RB = (uint32_t)a.RB;
        const uint32_t CT2a = (a.CT >> 1) & ~7u;
        if (!SHARED) {                              // one row block: no division
            rb = 0;
            ct2 = id;
        } else if (id < CT2a * RB) {
            const uint32_t xcd = id & 7u, slot = id >> 3;
            rb = slot % RB;
            ct2 = (slot / RB) * 8u + xcd;
        } else {
            const uint32_t t = id - CT2a * RB;
            rb = t % RB;
            ct2 = CT2a + t / RB;
        }
    };
    const int RT = (a.m + kTile - 1) / kTile;       // row tiles that exist in the workspace
    const int KB = a.KB;

    // ---- this wave's share of the loads of one stage (sources at k-block 0) ----
    // Waves 0-3 (the first wave of each SIMD) load the X tiles, from L2: wave w the DX planes
    // of row tile w of the row block (clamped to a row tile that exists; rows past m are
    // never used).  Waves 4-7 (the second of each SIMD) load the ciphertext tiles, from HBM:
    // waves 4 and 5 the planes of the first column tile (planes 0-3 and 4 .. DQ-1), waves 6
    // and 7 those of the second.  A load's source is the wave's buffer descriptor (base of
    // the tile's X or ciphertext region), the lane's 16 bytes, and a wave-uniform
    // offset: the operand tile's place at k-block 0 plus the carried k-block offset.  (A row
    // tile or column tile of planes spans KB * D KiB < 2^23 bytes.  Everything up to the first
    // loads is scalar work on the critical path of the launch: no divisions, and whatever the
    // loads do not need comes after them.)
    const uint32_t a_tile_bytes = (uint32_t)KB * DX * kTileBytes;     // one row tile, all k-blocks
    const uint32_t b_tile_bytes = (uint32_t)KB * DQ * kTileBytes;     // one column tile
    const bool loads_x = wave < 4;
    const uint32_t lane16 = (uint32_t)lane * 16u;
    constexpr int PH = (DQ + 1) / 2;                // planes of a column tile on its first wave
    static_assert(P_::MAXU == 4 && DX <= 4 && PH <= 4, "four load slots per wave and stage");
    const uint32_t src_step = (uint32_t)(loads_x ? DX : DQ) * kTileBytes;   // per k-block
    const uint32_t src_end = (uint32_t)KB * src_step;
    const uint32_t slot_step = loads_x ? P_::A_BYTES : P_::B_BYTES;
    const uint32_t slot_end = RING * slot_step;
    uint32_t dst[P_::MAXU];                         // the operand tile's byte offset in slot 0 of the LDS
    int n_loads;                                    // loads per stage
    {
        uint32_t first_tile;
        if (loads_x) {
            first_tile = (uint32_t)wave * DX;
            n_loads = DX;
        } else {
            const uint32_t c = (uint32_t)(wave >> 1) & 1u, hi = (uint32_t)wave & 1u;
            first_tile = (uint32_t)P_::A_TILES * RING + c * DQ + hi * PH;
            n_loads = hi ? DQ - PH : PH;
        }
#pragma unroll
        for (int u = 0; u < P_::MAXU; ++u) dst[u] = (first_tile + (uint32_t)u) * kTileBytes;
    }
    // Issue side of a tile: descriptor, the operand tiles' offsets at k-block 0, and the
    // wave-uniform state for the next stage to issue (byte offset of its k-block in the
    // source, byte offset of its slot in the ring; carried and wrapped, never recomputed).
    // Stage s of a tile is k-block (s + k_start) mod KB: the sum over k does not care about
    // the order, and workgroups that walk their (equally spaced) ciphertext regions in
    // lockstep would otherwise ask the same memory channels for data at the same moment.
    // The start depends on the column tile alone: row blocks that share a column tile walk
    // it together.
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t toff[P_::MAXU];                        // the operand tile's byte offset at k-block 0
    uint32_t src_off, slot_off;
    auto begin_tile = [&](uint32_t p, uint32_t ct2, uint32_t rb) {
        const uint4 *xd_p = b.prob[0].xd, *planes_p = b.prob[0].planes;
        if (!single) {
            xd_p = b.prob[p].xd;
            planes_p = b.prob[p].planes;
        }
        const unsigned char *const a_base =
            (const unsigned char *)xd_p + (size_t)rb * 4u * a_tile_bytes;
        const unsigned char *const b_base =
            (const unsigned char *)planes_p + (size_t)ct2 * 2u * b_tile_bytes;
        rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(loads_x ? a_base : b_base), 0, 0xffffffff,
                                                 0x00027000);
        uint32_t first_off;
        if (loads_x) {
            int r = wave;
            const int last = RT - 1 - (int)rb * 4;  // last row tile of the block that exists (>= 0)
            if (r > last) r = last;
            first_off = (uint32_t)r * a_tile_bytes;
        } else {
            const uint32_t c = (uint32_t)(wave >> 1) & 1u, hi = (uint32_t)wave & 1u;
            first_off = c * b_tile_bytes + hi * (PH * kTileBytes);
        }
#pragma unroll
        for (int u = 0; u < P_::MAXU; ++u) toff[u] = first_off + (uint32_t)u * kTileBytes;
        uint32_t k_start = ct2 - __umulhi(ct2, a.kb_magic) * (uint32_t)KB;   // ct2 mod KB
        if (k_start >= (uint32_t)KB) k_start -= (uint32_t)KB;
        src_off = k_start * src_step;
        slot_off = 0;
    };
    auto bump = [](uint32_t v, uint32_t step, uint32_t end) -> uint32_t {
        v += step;
        return v == end ? 0u : v;
    };
    // load u of the stage at the carried offsets
    auto issue_one = [&](auto u_c) {
        constexpr int u = decltype(u_c)::value;
        unsigned char *const d = lds + (dst[u] + slot_off);
        dma_tile<!SHARED>(rsrc, lane16, toff[u] + src_off, d);
    };
#define NIMBUS_NEXT_ISSUE()                                                   \
    do {                                                                      \
        src_off = bump(src_off, src_step, src_end);                           \
        slot_off = bump(slot_off, slot_step, slot_end);                       \
    } while (0)

    uint32_t tile = blockIdx.x, prob, ct2, rb;
    map_tile(tile, prob, ct2, rb);
    begin_tile(prob, ct2, rb);
    n_loads = __builtin_amdgcn_readfirstlane(n_loads);

    // One pass of this loop per tile.  The first stages of a tile other than the first are
    // in flight when its pass begins: they were issued in front of the epilogue of the tile
    // before it.
    for (bool first = true;; first = false) {
    v16i acc[ND];
    if (first) {
        // ---- up front: stages 0 .. LEAD-1 of the first tile ----
        // The accumulators are cleared between the stages: the memory pipeline takes the first
        // loads of a launch slowly (nothing is translated or cached yet), and the moves fill
        // the time the wave would spend waiting for it to accept the next one.
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
    } else {
#pragma unroll
        for (int d = 0; d < ND; ++d) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[d][r] = 0;
            tie_acc(acc[d]);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- what the first loads did not need ----
    const int rt = (int)rb * 4 + wr;                // this wave's row tile
    const bool active = FULL || rt < RT;            // wave-uniform
    // Loads and stores complete in the order they were issued, so the counted waits of the
    // loop would still be right with the epilogue's stores among the younger ones; waiting
    // for everything once (the loads have had the whole epilogue to land) keeps them simple.
    if (!first) wait_vmem<0>();
    // The column's ciphertext sum is needed after the loop; asked for now it costs two
    // registers, not a round trip to memory at the end.  An ordinary load: the compiler places
    // the wait for it at its first use, and the statements below that clobber memory keep the
    // load itself up here.  (One more load ahead of the loop's counted waits only makes them
    // wait for it too; it is the oldest but LEAD stages by then.)
    const uint64_t *colsum_p = b.prob[0].colsum;
    const uint64_t *mask_p = b.prob[0].mask;
    uint64_t *out_p = b.prob[0].out;
    if (!single) {
        colsum_p = b.prob[prob].colsum;
        mask_p = b.prob[prob].mask;
        out_p = b.prob[prob].out;
    }
    const uint64_t colsum_S =
        colsum_p[(ct2 * 2u + (uint32_t)wc) * kTile + (uint32_t)(lane & 31)];
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
            (void *)((const unsigned char *)mask_p + first), 0,
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
                        dma_tile<true>(rsrc_m, voff_m, soff_m, lds + dst_m);
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
                                dma_tile<!SHARED>(rsrc, lane16, toff[j] + src_off,
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
    } else if constexpr (PIPELINED) {
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
#undef NIMBUS_NEXT_READ
    // the last pipelined iteration has read a stage that does not exist into the other
    // operand set; nothing may reuse those registers before the reads are back
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

    // ---- the next tile's first stages, issued in front of this tile's epilogue ----
    // Every wave has the last stage in registers once all have passed the last barrier
    // (pipelined variants: the reads are waited for in front of it; the others read behind
    // it, so they meet once more here): the rings are free, and the loads have the whole
    // epilogue, which uses neither the rings nor the memory pipeline much, to land.
    const uint32_t next = tile + gridDim.x;
    const bool more = next < a.tiles;
    uint32_t next_prob = 0, next_ct2 = 0, next_rb = 0;
    if (more) {
        if constexpr (!PIPELINED) __builtin_amdgcn_s_barrier();
        map_tile(next, next_prob, next_ct2, next_rb);
        begin_tile(next_prob, next_ct2, next_rb);
#pragma unroll
        for (int st = 0; st < LEAD; ++st) {
            if (st < KB) {
                static_for<0, P_::MAXU>([&](auto u_c) {
                    if (decltype(u_c)::value < n_loads) issue_one(u_c);
                });
                NIMBUS_NEXT_ISSUE();
            }
        }
    }
    asm volatile("" ::: "memory");

    // ---- epilogue: rebuild, add the constant and the mask, reduce, store ----
    // (the lane number goes through an opaque copy: what the epilogue derives from it would
    // otherwise be computed once in front of all tiles and held in registers through the loop)
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    if (active)
        cop_epilogue<ND, FULL, MASKLDS>(
            acc, a, mask_p, a.prev, out_p, limb, colsum_S, rt * kTile + 4 * (lane_e >> 5),
            (ct2 * 2u + (uint32_t)wc) * kTile + (uint32_t)(lane_e & 31),
            lds + (MASKLDS ? P_::LDS_BYTES : 0) + (uint32_t)(wr * kTile + 4 * (lane_e >> 5)) * 512u +
                (uint32_t)(wc * kTile + (lane_e & 31)) * 8u);
    if (!more) break;
    tile = next;
    prob = next_prob;
    ct2 = next_ct2;
    rb = next_rb;
    }   // tiles
#undef NIMBUS_NEXT_ISSUE
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
// compute units of the current device (asked once per device)
static int compute_units()
{
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
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
    const hipError_t e =
        launch(prepare_planes_kernel<DQ>, dim3((unsigned)((total + 255) / 256)), dim3(256), stream,
               ctW, p.k, (uint32_t)p.C, p.N, p.L, p.limbs, KB, total, planes);
    if (e != hipSuccess) return e;
    return launch(column_sums_kernel, dim3((unsigned)((p.C + 255) / 256)), dim3(256), stream,
                  ctW, p.k, (uint32_t)p.C, p.N, p.L, p.limbs, colsum);
}

hipError_t launch_prepare(const Problem &p, const uint64_t *ctW, void *prepared,
                          hipStream_t stream)
{
    if (planes_q(p.q_bits_max) == 7) return prepare_impl<7>(p, ctW, prepared, stream);
    return prepare_impl<8>(p, ctW, prepared, stream);
}

template <int DX>
static hipError_t stage_impl(const Problem &p, int count, const uint64_t *const *X, int half_shift,
                             void *const *workspace, hipStream_t stream)
{
    const int KB = kblocks(p.k);
    const int RT = (p.m + kTile - 1) / kTile;
    const uint32_t xtotal = (uint32_t)RT * KB * 256;
    StagePtrs sp{};
    for (int i = 0; i < count; ++i) {
        sp.X[i] = X[i];
        sp.xd[i] = (uint32_t *)workspace[i];
    }
    return launch(x_planes_kernel<DX>, dim3((xtotal + 255) / 256, (uint32_t)count), dim3(256), stream,
                  sp, p.m, p.k, KB, xtotal, share_offset(p.x_bits, DX), half_shift);
}

// p.x_bits (<= 32) is the width of the half that is staged; half_shift is 0 or 32
hipError_t launch_stage_shares(const Problem &p, const uint64_t *X, int half_shift,
                               void *workspace, hipStream_t stream)
{
    return launch_stage_shares_batch(p, 1, &X, half_shift, &workspace, stream);
}

// the shares of count calls of the same shape in one launch
hipError_t launch_stage_shares_batch(const Problem &p, int count, const uint64_t *const *X,
                                     int half_shift, void *const *workspace, hipStream_t stream)
{
    if (count < 1 || count > kMaxBatch) return hipErrorInvalidValue;
    switch (planes_x(p.x_bits)) {
    case 2: return stage_impl<2>(p, count, X, half_shift, workspace, stream);
    case 3: return stage_impl<3>(p, count, X, half_shift, workspace, stream);
    default: return stage_impl<4>(p, count, X, half_shift, workspace, stream);
    }
}

// count problems of the same shape in one launch (count = 1: the ordinary call); the masks are
// all there or all null; prev only with count = 1
template <int DX, int DQ>
static hipError_t mfma_impl(const Problem &p, int count, const void *const *staged,
                            const void *const *prepared, const uint64_t *const *masks,
                            const uint64_t *prev, uint64_t *const *outs, hipStream_t stream)
{
    const int KB = kblocks(p.k);
    const uint32_t CT = (uint32_t)(p.C / kTile);
    const uint64_t *const mask = masks[0];

    MfmaArgs a{};
    fill_common_args(p, DX, mask, prev, outs[0], &a);
    BatchPtrs b{};
    for (int i = 0; i < count; ++i) {
        b.prob[i].xd = (const uint4 *)staged[i];
        b.prob[i].planes = (const uint4 *)prepared[i];
        b.prob[i].colsum = (const uint64_t *)((const char *)prepared[i] + (size_t)CT * KB * DQ * kTileBytes);
        b.prob[i].mask = masks[i];
        b.prob[i].out = outs[i];
    }
    b.count = (uint32_t)count;
    b.tiles_each = a.tiles;
    a.tiles *= (uint32_t)count;
    // One workgroup per compute unit at most (a compute unit holds one at a time anyway);
    // each walks the tiles id, id + grid, ...  A grid that is a multiple of 8 keeps a tile id's
    // XCD the same on every pass.
    uint32_t cus = (uint32_t)compute_units();
    if (cus >= 8) cus &= ~7u;
    const dim3 grid(a.tiles < cus ? a.tiles : cus);
    using P_ = Pipe<DX, DQ>;
    constexpr bool kCanMaskLds = P_::PIPELINED && P_::LDS_BYTES + kMaskTileBytes <= 160 * 1024;
    // mask tile in LDS: see the kernel; 128 rows of the mask must span less than 4 GB
    const bool mask_lds = kCanMaskLds && mask != nullptr && p.m % 128 == 0 &&
                          KB - P_::LEAD >= kMaskPhase && (uint64_t)p.C * 8u * 128u < (1ull << 32);
    const bool full = p.m % 128 == 0;
    auto launch = [&](auto full_c, auto masklds_c, auto shared_c) {
        return nimbus::launch(cop_mfma_kernel<DX, DQ, decltype(full_c)::value,
                                              decltype(masklds_c)::value, decltype(shared_c)::value>,
                              grid, dim3(512), stream, a, b);
    };
    using T = std::true_type;
    using F = std::false_type;
    if constexpr (kCanMaskLds) {
        if (mask_lds) return a.RB > 1 ? launch(T{}, T{}, T{}) : launch(T{}, T{}, F{});
    }
    if (a.RB > 1) return full ? launch(T{}, F{}, T{}) : launch(F{}, F{}, T{});
    return full ? launch(T{}, F{}, F{}) : launch(F{}, F{}, F{});
}

hipError_t launch_cop_mfma(const Problem &p, const void *staged, const void *prepared,
                           const uint64_t *mask, const uint64_t *prev, uint64_t *out,
                           hipStream_t stream)
{
    return launch_cop_mfma_batch(p, 1, &staged, &prepared, &mask, prev, &out, stream);
}

hipError_t launch_cop_mfma_batch(const Problem &p, int count, const void *const *staged,
                                 const void *const *prepared, const uint64_t *const *masks,
                                 const uint64_t *prev, uint64_t *const *outs, hipStream_t stream)
{
    if (count < 1 || count > kMaxBatch) return hipErrorInvalidValue;
    const int DX = planes_x(p.x_bits), DQ = planes_q(p.q_bits_max);
#define NIMBUS_CASE(dx, dq) \
    if (DX == dx && DQ == dq) \
        return mfma_impl<dx, dq>(p, count, staged, prepared, masks, prev, outs, stream);
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
