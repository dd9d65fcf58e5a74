// Matrix-core (int8 MFMA) kernel for the COP accumulation on the CANONICAL layout, gfx950:
// nimbus_cop_matmul without any setup pass.  Same contraction and same epilogue as the kernel
// for prepared weights (cop_mfma.hip; Algorithm 1 step 2 + step 4 of the paper), but both
// operands arrive as 64-bit words and are split into signed byte planes inside the loop:
//
//   ciphertext words  ctW[k][C]: a 32 x 64 tile per k-block (16 KB) comes into a ring of raw
//       tiles in LDS by direct-to-LDS loads, three k-blocks ahead; one k-block ahead of its use
//       every thread takes four words of one column (four consecutive k), recodes them into
//       signed bytes (digits of the residue c itself: unlike the setup pass of the other
//       kernel it does not centre first, which would cost five vector instructions a word)
//       and writes one 32-bit word (four k-slots) into each of the DQ operand tiles of that
//       column tile;
//   shares  X[m][k]: a 128 x 32 tile per k-block comes from L2 into registers, one k-block
//       ahead; every thread turns 2 x 4 consecutive k of one row into one word per plane.
//
// The operand tiles in LDS have the register order of the instruction, exactly as the setup
// pass of the other kernel would have left them in memory, so the products are the same
// v_mfma_i32_32x32x32_i8 sequence: 8 waves, wave (wr, wc) owns 32 rows x 32 columns, DX * DQ
// instructions per k-block into DX + DQ - 1 diagonal accumulators.  The column sums S that the
// share offset OFFX needs (x = x' + OFFX) are gathered on the way: every thread adds up the
// words it converts, the partial sums meet in LDS after the loop.
//
// One barrier per k-block: it publishes the operand tiles of block s (written during block
// s - 1) and the raw tile of block s + 1, and it frees the operand buffer of block s - 1 and
// the raw slot of block s for the loads of block s + 3.
#include "cop_mfma_common.hpp"

namespace nimbus {

struct CanonArgs {
    MfmaArgs e;               // sizes, tile mapping, OFFX and the epilogue's constants
    const uint64_t *X;        // [m][k]
    const uint64_t *ctW;      // [k][C]
    int k;
    LimbTable limbs;          // reduction of the column sums
};

template <int OFF>
__device__ __forceinline__ uint64_t lds_read_b64(uint32_t addr)
{
    uint64_t r;
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
    return r;
}
template <int OFF>
__device__ __forceinline__ void lds_write_b32(uint32_t addr, uint32_t v)
{
    asm volatile("ds_write_b32 %0, %1 offset:%2" ::"v"(addr), "v"(v), "n"(OFF) : "memory");
}
__device__ __forceinline__ void tie64(uint64_t &x) { asm volatile("" : "+v"(x)); }

// bytes (a0 a1 a2 a3), (b0 ..), (c0 ..), (d0 ..) -> (a0 b0 c0 d0), (a1 b1 c1 d1), ...
// (a 4 x 4 byte transpose: word j of the result holds byte j of each input)
__device__ __forceinline__ void transpose4(uint32_t a, uint32_t b, uint32_t c, uint32_t d,
                                           uint32_t (&t)[4])
{
    // v_perm_b32(hi, lo, sel): byte i of the result is byte sel_i of the 8 bytes {hi, lo}
    const uint32_t ab_lo = __builtin_amdgcn_perm(b, a, 0x05010400u);   // a0 b0 a1 b1
    const uint32_t ab_hi = __builtin_amdgcn_perm(b, a, 0x07030602u);   // a2 b2 a3 b3
    const uint32_t cd_lo = __builtin_amdgcn_perm(d, c, 0x05010400u);   // c0 d0 c1 d1
    const uint32_t cd_hi = __builtin_amdgcn_perm(d, c, 0x07030602u);   // c2 d2 c3 d3
    t[0] = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x05040100u);           // a0 b0 c0 d0
    t[1] = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x07060302u);           // a1 b1 c1 d1
    t[2] = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x05040100u);
    t[3] = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x07060302u);
}

// FULL: m is a multiple of 128.  SHARED: several row blocks per column tile (m > 128); they
// start at the same k-block and load the ciphertext without the streaming hint, so that the
// tile is found in the L2 of their XCD by all but the first.
// CENTRE: the ciphertext digits are those of the centred residue (c or c - q) instead of the
// residue itself.  Needed when a residue can exceed what DQ signed digits express,
// 127 (256^DQ - 1) / 255 (moduli within half a percent of 2^(8 DQ - 1)); costs five vector
// instructions a word.
template <int DX, int DQ, bool FULL, bool SHARED, bool CENTRE>
__global__ __launch_bounds__(512, 1) void cop_canon_kernel(const CanonArgs ca)
{
    const MfmaArgs &a = ca.e;
    constexpr int ND = DX + DQ - 1;
    constexpr int A_BYTES = 4 * DX * kTileBytes, B_BYTES = 2 * DQ * kTileBytes;
    constexpr int STAGE = A_BYTES + B_BYTES;            // operand tiles of one k-block
    // raw ciphertext tile: 16 loads of 1 KB (two k-rows of 64 words each); the four k-rows
    // 4g .. 4g+3 of k-group g take 2 KB, followed by 128 bytes of padding, so that
    // neighbouring k-groups, which the two halves of a wave read at once, start in different
    // halves of the banks
    constexpr int RAW_GROUP = 2 * kTileBytes + 128;
    constexpr int RAW_SLOT = 8 * RAW_GROUP, RAW_RING = 3;
    constexpr int RAW0 = 2 * STAGE;
    constexpr int LDS_BYTES = RAW0 + RAW_RING * RAW_SLOT;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    static_assert(64 * 8 * 16 <= RAW_RING * RAW_SLOT, "the column sums reuse the raw ring");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // 0..7
    const int wr = wave >> 1, wc = wave & 1;

    // workgroup -> (64-column tile, row block), as in the kernel for prepared weights
    uint32_t ct2, rb;
    {
        const uint32_t id = blockIdx.x;
        const uint32_t RB = (uint32_t)a.RB;
        const uint32_t CT2a = (a.CT >> 1) & ~7u;
        if (!SHARED) {
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
    }
    const int RT = (a.m + kTile - 1) / kTile;
    const int rt = (int)rb * 4 + wr;
    const bool active = FULL || rt < RT;            // this wave has rows (wave-uniform)
    const int KB = a.KB;
    const uint32_t K = (uint32_t)ca.k, C = a.C;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(NIMBUS_AS3 void *)&lds[0];

    // ---- ciphertext side: raw tile loads and this thread's conversion item ----
    // load p of a stage (0 <= p < 16) moves k-rows 2p and 2p+1 of the tile: lanes 0-31 the 64
    // words of row 2p (16 bytes = two columns per lane), lanes 32-63 those of row 2p+1.  Wave w
    // issues loads w and w + 8.  Rows past k read as zero (the descriptor ends with ctW), and a
    // zero word recodes to zero digits: the padding of the last k-block costs nothing.
    const uint64_t ct_first = (uint64_t)ct2 * 64u * 8u;
    const __amdgpu_buffer_rsrc_t rsrc_ct = __builtin_amdgcn_make_buffer_rsrc(
        (void *)((const unsigned char *)ca.ctW + ct_first), 0,
        (uint32_t)((uint64_t)K * C * 8u - ct_first), 0x00027000);
    const uint32_t voff_ct = (uint32_t)(lane >> 5) * C * 8u + (uint32_t)(lane & 31) * 16u;
    const uint32_t row_bytes = C * 8u;
    uint32_t ct_src[2], ct_dst[2];                  // wave-uniform: source offset in the k-block, place in the slot
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t p = (uint32_t)wave + 8u * (uint32_t)i;
        ct_src[i] = 2u * p * row_bytes;
        ct_dst[i] = (uint32_t)RAW0 + (p >> 1) * RAW_GROUP + (p & 1u) * kTileBytes;
    }
    // conversion item: column c of the tile (16 columns per wave), k-group g (k = 4g .. 4g+3)
    const uint32_t cv_c = 16u * ((uint32_t)wave & 3u) + ((uint32_t)lane & 15u);
    const uint32_t cv_g = 4u * ((uint32_t)wave >> 2) + ((uint32_t)lane >> 4);
    const uint32_t cv_raw = lds0 + (uint32_t)RAW0 + cv_g * RAW_GROUP + cv_c * 8u;
    // its word in the operand tiles: column tile cv_c / 32, lane slot (cv_c % 32) + 32 (g / 4),
    // word g % 4; plane b follows at b KB
    const uint32_t cv_out = lds0 + (uint32_t)A_BYTES + (cv_c >> 5) * (DQ * kTileBytes) +
                            ((cv_c & 31u) + 32u * (cv_g >> 2)) * 16u + (cv_g & 3u) * 4u;
    // modulus of the item's column (16 aligned columns lie in one limb: N >= 32)
    uint64_t cv_q = 0;
    if constexpr (CENTRE) {
        const uint32_t blk = ((ct2 * 2u + (((uint32_t)wave & 3u) >> 1)) * kTile) >> a.log_n;
        uint32_t l = a.L == 1 ? 0u : blk - (uint32_t)a.L * __umulhi(blk, a.l_magic);
        l = __builtin_amdgcn_readfirstlane(l);
        cv_q = a.q[l];
    }
    const uint64_t cv_half = (cv_q - 1) >> 1;
    uint64_t bias = 0;                              // 0x80 in each of the DQ low bytes
#pragma unroll
    for (int d = 0; d < DQ; ++d) bias |= (uint64_t)0x80 << (8 * d);
    // sums of the lower and of the upper halves of the words this thread converts (one
    // 32 x 32 + 64-bit multiply-add by one each: k / 8 words of 32 bits cannot overflow 64)
    uint64_t sum_lo = 0, sum_hi = 0;

    // ---- share side: two items per thread, item i: 16 rows x 4 k-quads per wave ----
    // item t = 2 wave + i: rows 16 (t % 8) + lane / 4, k-quad 4 (t / 8) + lane % 4 (k = 4 kq .. +3)
    const uint64_t x_first = (uint64_t)rb * 128u * K * 8u;
    const uint64_t x_left = (uint64_t)a.m * K * 8u - x_first;
    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
        (void *)((const unsigned char *)ca.X + x_first), 0,
        x_left > 0xffffffffull ? 0xffffffffu : (uint32_t)x_left, 0x00027000);
    uint32_t voff_x[2], x_out[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t t = 2u * (uint32_t)wave + (uint32_t)i;
        const uint32_t r = 16u * (t & 7u) + ((uint32_t)lane >> 2);
        const uint32_t kq = 4u * (t >> 3) + ((uint32_t)lane & 3u);
        voff_x[i] = r * K * 8u + kq * 32u;
        // row tile r / 32, lane slot (r % 32) + 32 (kq / 4), word kq % 4; plane a at a KB
        x_out[i] = lds0 + (r >> 5) * (DX * kTileBytes) + ((r & 31u) + 32u * (kq >> 2)) * 16u +
                   (kq & 3u) * 4u;
    }

    // stage s is k-block (s + k_start) mod KB (column tiles start at different k-blocks)
    uint32_t k_start = ct2 - __umulhi(ct2, a.kb_magic) * (uint32_t)KB;
    if (k_start >= (uint32_t)KB) k_start -= (uint32_t)KB;
    uint32_t kb_issue = k_start;                    // k-block of the next stage whose loads go out
    auto next_kb = [&](uint32_t kb) -> uint32_t { return kb + 1 == (uint32_t)KB ? 0u : kb + 1; };
    uint32_t raw_issue = 0;                         // raw slot of that stage (0 .. RAW_RING-1)
    auto issue_raw = [&]() {                        // both loads of this wave for the stage
#pragma unroll
        for (int i = 0; i < 2; ++i)
            // (the whole offset goes into the per-lane operand: that is the one the range
            // check of the descriptor looks at, and rows past k must read as zero)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rsrc_ct, (NIMBUS_AS3 void *)(lds + (ct_dst[i] + raw_issue * RAW_SLOT)), 16,
                voff_ct + (ct_src[i] + kb_issue * 32u * row_bytes), 0, 0, SHARED ? 0 : 2);
        kb_issue = next_kb(kb_issue);
        raw_issue = raw_issue + 1 == RAW_RING ? 0u : raw_issue + 1;
    };
    uint32_t kb_x = k_start;                        // k-block of the next share loads
    v4i xr[2][2];                                   // raw shares: [item][half of the 32 bytes]
    auto load_x = [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t at = voff_x[i] + kb_x * 256u;
            xr[i][0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, at, 0, 0);
            xr[i][1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, at + 16u, 0, 0);
        }
        kb_x = next_kb(kb_x);
    };

    // conversion of one stage, in pieces that the loop places between its matrix-core
    // instructions: raw slot `rs`, operand buffer `ob`
    uint64_t cw[4];
    auto ct_read = [&](uint32_t rs) {
        const uint32_t base = cv_raw + rs * RAW_SLOT;
        cw[0] = lds_read_b64<0>(base);
        cw[1] = lds_read_b64<512>(base);
        cw[2] = lds_read_b64<1024>(base);
        cw[3] = lds_read_b64<1536>(base);
    };
    auto ct_recode = [&]() {                        // after the LDS wait
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            tie64(cw[j]);
            const uint64_t c = cw[j];
            asm("v_mad_u64_u32 %0, vcc, %1, 1, %0" : "+v"(sum_lo) : "v"((uint32_t)c) : "vcc");
            asm("v_mad_u64_u32 %0, vcc, %1, 1, %0" : "+v"(sum_hi) : "v"((uint32_t)(c >> 32)) : "vcc");
            // signed base-256 digits of the residue, centred first where it has to be:
            // c' + 0x80..80 has the bytes digit + 128, and flipping bit 7 of each gives the
            // digits as signed bytes
            const uint64_t cc = CENTRE && c > cv_half ? c - cv_q : c;  // two's complement of c'
            cw[j] = (cc + bias) ^ bias;
        }
    };
    auto ct_write = [&](uint32_t ob) {
        const uint32_t base = cv_out + ob * STAGE;
        uint32_t t[4];
        transpose4((uint32_t)cw[0], (uint32_t)cw[1], (uint32_t)cw[2], (uint32_t)cw[3], t);
        lds_write_b32<0 * kTileBytes>(base, t[0]);
        lds_write_b32<1 * kTileBytes>(base, t[1]);
        lds_write_b32<2 * kTileBytes>(base, t[2]);
        lds_write_b32<3 * kTileBytes>(base, t[3]);
        transpose4((uint32_t)(cw[0] >> 32), (uint32_t)(cw[1] >> 32), (uint32_t)(cw[2] >> 32),
                   (uint32_t)(cw[3] >> 32), t);
        lds_write_b32<4 * kTileBytes>(base, t[0]);
        lds_write_b32<5 * kTileBytes>(base, t[1]);
        lds_write_b32<6 * kTileBytes>(base, t[2]);
        if constexpr (DQ == 8) lds_write_b32<7 * kTileBytes>(base, t[3]);
    };
    auto x_write = [&](uint32_t ob, auto i_c) {     // item i: regs -> DX plane words
        constexpr int i = decltype(i_c)::value;
        const uint32_t base = x_out[i] + ob * STAGE;
        uint32_t t[4];
        // flipping bit 7 of the shifted bytes turns them into the digits byte - 128
        transpose4((uint32_t)xr[i][0].x ^ a.offx, (uint32_t)xr[i][0].z ^ a.offx,
                   (uint32_t)xr[i][1].x ^ a.offx, (uint32_t)xr[i][1].z ^ a.offx, t);
        lds_write_b32<0 * kTileBytes>(base, t[0]);
        lds_write_b32<1 * kTileBytes>(base, t[1]);
        if constexpr (DX >= 3) lds_write_b32<2 * kTileBytes>(base, t[2]);
        if constexpr (DX >= 4) lds_write_b32<3 * kTileBytes>(base, t[3]);
    };

    // ---- prologue: raw tiles of stages 0 .. 2 and the shares of stage 0 on their way,
    // accumulators cleared, stage 0 converted into operand buffer 0 ----
    issue_raw();
    load_x();
    if (KB > 1) issue_raw();
    if (KB > 2) issue_raw();
    v16i acc[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[d][r] = 0;
        tie_acc(acc[d]);
    }
    // this wave's raw loads of stage 0 are older than its 4 share loads and 2 loads per later stage
    wait_vmem_n(4 + 2 * (KB > 2 ? 2 : KB - 1));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    ct_read(0);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    ct_recode();
    ct_write(0);
    x_write(0, std::integral_constant<int, 0>{});
    x_write(0, std::integral_constant<int, 1>{});

    // ---- the loop ----
    const uint32_t laneA = lds0 + (uint32_t)(wr * DX) * kTileBytes + (uint32_t)lane * 16u;
    const uint32_t laneB = lds0 + (uint32_t)A_BYTES + (uint32_t)(wc * DQ) * kTileBytes +
                           (uint32_t)lane * 16u;
    constexpr int NPOS = DX * DQ;
    uint32_t ob = 0, rs = 1;                        // operand buffer of stage s, raw slot of stage s + 1
    for (int s = 0; s < KB; ++s) {
        const bool more = s + 1 < KB;               // stage s + 1 exists: convert it during this block
        // operand words of stage s written, raw tile of stage s + 1 landed (younger: the two
        // loads of stage s + 2), then the barrier
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (s + 3 < KB) wait_vmem<2>();             // steady state: stage s + 2 may be in flight
        else wait_vmem<0>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        v4i xa[DX], xb[DQ];
        if (active) {
            const uint32_t pa = laneA + ob * STAGE, pb = laneB + ob * STAGE;
            static_for<0, DX>([&](auto d_c) {
                constexpr int d = decltype(d_c)::value;
                xa[d] = lds_read_b128<d * kTileBytes>(pa);
            });
            static_for<0, DQ>([&](auto d_c) {
                constexpr int d = decltype(d_c)::value;
                xb[d] = lds_read_b128<d * kTileBytes>(pb);
            });
        }
        if (more) {
            load_x();                               // shares of stage s + 1 (from L2)
            ct_read(rs);                            // raw words of stage s + 1
        }
        if (s + 3 < KB) issue_raw();                // stage s + 3 into the slot stage s has left
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (active) {
#pragma unroll
            for (int d = 0; d < DX; ++d) tie(xa[d]);
#pragma unroll
            for (int d = 0; d < DQ; ++d) tie(xb[d]);
        }
        const uint32_t nb = ob ^ 1u;                // operand buffer of stage s + 1
        static_for<0, NPOS>([&](auto i_c) {
            constexpr int i = decltype(i_c)::value;
            constexpr int dx = i / DQ, dq = i % DQ;
            if (active) {
                tie(xa[dx]);
                tie(xb[dq]);
                acc[dx + dq] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xa[dx], xb[dq], acc[dx + dq],
                                                                     0, 0, 0);
                tie_acc(acc[dx + dq]);
            }
            if constexpr (i == NPOS / 8) { if (more) ct_recode(); }
            if constexpr (i == NPOS / 2) { if (more) ct_write(nb); }
            if constexpr (i == (3 * NPOS) / 4) { if (more) x_write(nb, std::integral_constant<int, 0>{}); }
            if constexpr (i == (7 * NPOS) / 8) { if (more) x_write(nb, std::integral_constant<int, 1>{}); }
        });
        asm volatile("" ::: "memory");
        ob = nb;
        rs = rs + 1 == RAW_RING ? 0u : rs + 1;
    }

    // ---- column sums: the eight k-groups of a column meet in LDS (over the raw ring, which
    // nobody reads any more once every wave is past the loop) ----
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    {
        const uint32_t at = lds0 + (uint32_t)RAW0 + (cv_c * 8u + cv_g) * 16u;
        asm volatile("ds_write_b64 %0, %1\n\tds_write_b64 %0, %2 offset:8"
                     ::"v"(at), "v"(sum_lo), "v"(sum_hi) : "memory");
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (!active) return;
    uint32_t limb;
    {
        const uint32_t blk = ((ct2 * 2u + (uint32_t)wc) * kTile) >> a.log_n;
        limb = a.L == 1 ? 0u : blk - (uint32_t)a.L * __umulhi(blk, a.l_magic);
        limb = __builtin_amdgcn_readfirstlane(limb);
    }
    uint64_t colsum_S;
    {
        const uint32_t at = lds0 + (uint32_t)RAW0 + ((uint32_t)(wc * kTile + (lane & 31)) * 8u) * 16u;
        uint64_t lows = 0, highs = 0;               // each below 2^32 k
        static_for<0, 8>([&](auto g_c) {
            constexpr int g = decltype(g_c)::value;
            uint64_t plo, phi;
            asm volatile("ds_read_b64 %0, %2 offset:%3\n\tds_read_b64 %1, %2 offset:%4\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(plo), "=&v"(phi) : "v"(at), "n"(g * 16), "n"(g * 16 + 8) : "memory");
            lows += plo;
            highs += phi;
        });
        uint64_t lo = lows, hi = 0;                 // lows + 2^32 highs in 128 bits
        add128(hi, lo, highs >> 32, highs << 32);
        colsum_S = barrett128(hi, lo, ca.limbs.limb[limb]);      // k * q < 2^(b+63)
    }
    cop_epilogue<ND, FULL, false>(acc, a, a.mask, nullptr, a.out, limb, colsum_S, rt * kTile + 4 * (lane >> 5),
                                  (ct2 * 2u + (uint32_t)wc) * kTile + (uint32_t)(lane & 31), nullptr);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
// DQ signed digits express the values up to 127 (256^DQ - 1) / 255: is there a limb whose
// residues can be larger?
static bool needs_centring(const Problem &p, int DQ)
{
    uint64_t top = 0;
    for (int d = 0; d < DQ; ++d) top = top * 256u + 127u;
    for (int l = 0; l < p.L; ++l)
        if (p.limbs.limb[l].q - 1 > top) return true;
    return false;
}

bool canon_supported(const Problem &p)
{
    if (p.x_bits > 32 || !mfma_supported(p)) return false;
    // where the digits stand for the residues themselves, not the centred ones, the sums are
    // twice as large and the multiple of q that makes them non-negative is one bit longer; the
    // value reduced in the epilogue must stay below 2^47 q all the same
    if (!needs_centring(p, planes_q(p.q_bits_max)) && bias_shift(p) + 3 > 47) return false;
    // four share planes times eight ciphertext planes: eleven accumulator tiles and the
    // conversion's registers do not fit one wave
    if (planes_x(p.x_bits) == 4 && planes_q(p.q_bits_max) == 8) return false;
    // 32-bit offsets inside the buffer descriptors: the whole of ctW, and the 128 rows of X of
    // a row block
    if ((uint64_t)p.k * p.C * 8u >= (1ull << 32)) return false;
    if ((uint64_t)p.k * 8u * 128u >= (1ull << 32)) return false;
    return true;
}

template <int DX, int DQ>
static hipError_t canon_impl(const Problem &p, const uint64_t *X, const uint64_t *ctW,
                             const uint64_t *mask, uint64_t *out, hipStream_t stream)
{
    CanonArgs ca{};
    const bool centre = needs_centring(p, DQ);
    fill_common_args(p, DX, mask, nullptr, out, &ca.e, centre ? 0 : 1);
    ca.X = X;
    ca.ctW = ctW;
    ca.k = p.k;
    ca.limbs = p.limbs;
    const dim3 grid((ca.e.CT / 2) * (uint32_t)ca.e.RB);
    const bool full = p.m % 128 == 0, shared = ca.e.RB > 1;
    auto go = [&](auto full_c, auto shared_c, auto centre_c) {
        return launch(cop_canon_kernel<DX, DQ, decltype(full_c)::value, decltype(shared_c)::value,
                                       decltype(centre_c)::value>,
                      grid, dim3(512), stream, ca);
    };
    using T = std::true_type;
    using F = std::false_type;
    if constexpr (DQ == 7) {                        // (eight digits express every q < 2^62)
        if (centre) {
            if (full) return shared ? go(T{}, T{}, T{}) : go(T{}, F{}, T{});
            return shared ? go(F{}, T{}, T{}) : go(F{}, F{}, T{});
        }
    }
    if (full) return shared ? go(T{}, T{}, F{}) : go(T{}, F{}, F{});
    return shared ? go(F{}, T{}, F{}) : go(F{}, F{}, F{});
}

hipError_t launch_cop_canon(const Problem &p, const uint64_t *X, const uint64_t *ctW,
                            const uint64_t *mask, uint64_t *out, hipStream_t stream)
{
    const int DX = planes_x(p.x_bits), DQ = planes_q(p.q_bits_max);
#define NIMBUS_CASE(dx, dq) \
    if (DX == dx && DQ == dq) return canon_impl<dx, dq>(p, X, ctW, mask, out, stream);
    NIMBUS_CASE(2, 7)
    NIMBUS_CASE(3, 7)
    NIMBUS_CASE(4, 7)
    NIMBUS_CASE(2, 8)
    NIMBUS_CASE(3, 8)
#undef NIMBUS_CASE
    return hipErrorInvalidValue;
}

}  // namespace nimbus
