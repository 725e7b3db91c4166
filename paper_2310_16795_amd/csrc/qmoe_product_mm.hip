// Kernels built on the ring decoder: the matrix-core product for crowded experts
// (Section 5.3 of the paper proposes decoding once for several tokens) and the
// decompression of whole matrices (Section 4.3.3 mentions it as a variant).
#include "qmoe_dev.h"

namespace qmoe {
namespace {

// ---------------------------------------------------------------- matrix-core product for crowded experts
//
// An expert with many tokens is a dense contraction once its ternary weights are
// in hand: y[token][row] = sum_k x[token][k] * W[row][k].  The scalar kernel
// would decode the matrix again for every few tokens; this one decodes it once per
// tile of up to 64 tokens.  A wavefront owns 64 rows (one lane per row) and walks
// the columns 64 at a time.  Every lane keeps a ring of 128 one-byte columns of its
// row in LDS and decodes its codewords into it sequentially, as far ahead as the
// ring allows (so the lanes of a wavefront, whose codewords end at different
// columns, seldom wait for each other); then the wavefront multiplies the 64
// columns that are complete, for the 64 rows its lanes decoded, with the tokens'
// activations on the matrix cores, fp32 accumulators in registers.  The
// ring holds the weights as the high byte of bf16 +-2.0 (0x40 / 0xC0, low byte
// zero), expanded to bf16 by a byte permute when a fragment is read; the factor 2
// is taken out again, exactly, when a row is written.
// Only device-order streams (whole table in LDS) take this path.

constexpr int kMmKc = 64;                      // columns per step
constexpr int kMmRing = 2 * kMmKc;             // columns a lane's ring holds
constexpr int kMmAhead = kMmRing - 28 - 1;     // a codeword may start this far past the step's first column (its run then ends
                                               // below column kc + 128, the first one that shares a ring byte with the step)
constexpr int kMmWRowBytes = kMmRing + 16;     // 36 banks per row: 16 consecutive rows read 16 bytes each (two lanes, 8 bytes apiece) without conflict

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));


// eight ring bytes (high bytes of bf16) -> eight bf16
__device__ __forceinline__ bf16x8 mm_expand(uint32_t d0, uint32_t d1)
{
    u32x4 o;
    o.x = __builtin_amdgcn_perm(0u, d0, 0x010c000cu);
    o.y = __builtin_amdgcn_perm(0u, d0, 0x030c020cu);
    o.z = __builtin_amdgcn_perm(0u, d1, 0x010c000cu);
    o.w = __builtin_amdgcn_perm(0u, d1, 0x030c020cu);
    bf16x8 r;
    __builtin_memcpy(&r, &o, 16);
    return r;
}

// Asymmetric grid: the ring holds byte selectors (0: zero, 2: w_max, 6: w_min) and eight of
// them pick the row's own bf16 grid points out of lo = w_max << 16, hi = w_min << 16 (bytes
// 0..3 of the permute's source are lo, 4..7 hi; selector b takes the value's low byte,
// b + 1 its high byte).
__device__ __forceinline__ bf16x8 mm_expand_minmax(uint32_t d0, uint32_t d1, uint32_t hi, uint32_t lo)
{
    u32x4 o;
    o.x = __builtin_amdgcn_perm(hi, lo, __builtin_amdgcn_perm(0u, d0, 0x01010000u) + 0x01000100u);
    o.y = __builtin_amdgcn_perm(hi, lo, __builtin_amdgcn_perm(0u, d0, 0x03030202u) + 0x01000100u);
    o.z = __builtin_amdgcn_perm(hi, lo, __builtin_amdgcn_perm(0u, d1, 0x01010000u) + 0x01000100u);
    o.w = __builtin_amdgcn_perm(hi, lo, __builtin_amdgcn_perm(0u, d1, 0x03030202u) + 0x01000100u);
    bf16x8 r;
    __builtin_memcpy(&r, &o, 16);
    return r;
}

using gw_u64 = __attribute__((address_space(1))) unsigned long long *;
using gw_u32x4 = __attribute__((address_space(1))) u32x4 *;
using lw_u8 = __attribute__((address_space(3))) unsigned char *;
using lw_u64 = __attribute__((address_space(3))) unsigned long long *;
using lw_u32x4 = __attribute__((address_space(3))) u32x4 *;
using lp_u64 = const __attribute__((address_space(3))) unsigned long long *;
using lp_u32x4 = const __attribute__((address_space(3))) u32x4 *;
using lp_i32 = const __attribute__((address_space(3))) int *;
using lp_f32 = const __attribute__((address_space(3))) float *;

// ---- the ring decoder shared by the matrix-core product and the decompression kernel ----
//
// One lane = one row.  A lane's codewords pass through a window of two 16-byte pieces (sixteen
// codewords) in LDS, the next piece is in flight in a register; the codeword two places ahead
// is read from the window and the table entry one place ahead is looked up while the current
// entry is applied.  Applying an entry is three one-byte stores into the lane's ring of 128
// columns: field z goes to ring column (column + position) mod 128 with the value bits of the
// field shifted to the top of the byte (0x40: +2.0, 0xC0: -2.0 as the high byte of bf16) or, for
// the asymmetric grid, as they are (byte selectors 2 / 6); an unused field (0) comes first and
// writes its zero at the run's first column before any real weight of the same run.
//
// (A struct of plain scalars and free functions that are always inlined: the state stays in
// registers.)
constexpr int kMmWinBytes = 40;   // a lane's window: two 16-byte pieces, padded so that the 64 slots spread over the banks

struct RingDecoder {
    uint32_t left;              // codewords to go
    uint32_t ci;                // index of the next codeword, counted from the lane's first piece
    uint32_t wbase;             // index of the first codeword of the window's first piece (a multiple of 8)
    uint32_t pos8;              // 8 * (column where the next run starts)
    uint32_t ent, ent_n, flips_n, c1, c2;  // the pipeline: entry of codeword ci, entry of ci + 1 as read and the
                                           // sign flips of its code, codes of ci + 1 and ci + 2
    uintptr_t pp, last, pstr;   // first piece of the window, the lane's last piece, bytes from a piece to the next
    u32x4 fut;                  // the piece after the window, in flight
    uint32_t wrow, slot;        // LDS byte addresses of the lane's ring and window
};

__device__ __forceinline__ u32x4 ring_piece_at(const RingDecoder &d, uintptr_t at)
{
    // pieces past the lane's last one re-read the last (never used: `left` runs out first)
    return *(gp_u32x4)(at < d.last ? at : d.last);
}

__device__ __forceinline__ void ring_store_piece(const RingDecoder &d, uint32_t half_bytes, const u32x4 &v)
{
    lw_u64 w = (lw_u64)(uintptr_t)(d.slot + half_bytes);
    w[0] = (unsigned long long)v.x | ((unsigned long long)v.y << 32);
    w[1] = (unsigned long long)v.z | ((unsigned long long)v.w << 32);
}

__device__ __forceinline__ uint32_t ring_code_at(const RingDecoder &d, uint32_t i)
{
    return (uint32_t)(*(lp_u16)(uintptr_t)(d.slot + 2u * (i & 15u)));
}

__device__ __forceinline__ uint32_t ring_entry_index(uint32_t code, uint32_t n_groups, uint32_t n_order)
{
    return min(max(code >> 2, __builtin_elementwise_sub_sat(code, 3u * n_groups)), n_order - 1u);
}

// The lane's row (none: an empty stream), its window filled, its ring cleared.
__device__ __forceinline__ void ring_setup(RingDecoder &d, const qmoe_matrix &M, int row, bool row_live, uint32_t wrow,
                                           uint32_t slot)
{
    const RowStream rst = row_stream(M, row, row_live);
    d.left = rst.left;
    d.pp = rst.pp;
    d.last = rst.last;
    d.pstr = rst.pstride;
    d.ci = rst.sub;
    d.wrow = wrow;
    d.slot = slot;
    {
        const u32x4 p0 = ring_piece_at(d, d.pp), p1 = ring_piece_at(d, d.pp + d.pstr);
        ring_store_piece(d, 0u, p0);
        ring_store_piece(d, 16u, p1);
    }
    d.fut = ring_piece_at(d, d.pp + 2u * d.pstr);
    d.wbase = 0;
    d.pos8 = 0;
#pragma unroll
    for (int i = 0; i < kMmRing / 8; i++) ((lw_u64)(uintptr_t)wrow)[i] = 0ull;
}

// Fill the pipeline.  Nothing is in flight afterwards, so that the wait at the top of a round is
// for the two reads of the round before and not for the three stores issued after them.
__device__ __forceinline__ void ring_prime(RingDecoder &d, lp_u32 table, uint32_t n_groups, uint32_t n_order)
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    d.c1 = ring_code_at(d, d.ci + 1u);
    d.c2 = ring_code_at(d, d.ci + 2u);
    d.ent = order_entry(table, ring_code_at(d, d.ci), n_groups, n_order);
    d.ent_n = table[ring_entry_index(d.c1, n_groups, n_order)];
    d.flips_n = order_flips(d.c1);
    asm volatile("" : "+v"(d.ent_n), "+v"(d.c1), "+v"(d.c2), "+v"(d.ent));
}

// Decode until every lane of the wavefront has passed column kc + 64.  A lane that is there
// already keeps going as long as its next run starts at most kMmAhead columns past kc (its run
// then ends below column kc + 128, the first one that shares a ring byte with the step), so
// the lanes of a wavefront, whose codewords end at different columns, seldom wait for each
// other.  `after_wait` runs once, right after the step's wait for global memory: the place
// to issue loads that should stay in flight for a whole step.
//
// The pipeline: nothing that was just read is used in the round that reads it (a select or a
// sign flip on a fresh value would make the wavefront wait for it on the spot): a round's two
// reads are issued first, unconditional, from addresses chosen so that a lane that sat out
// reads again what it already holds, and are used a round later; the entry of ci + 1 is kept
// as read, next to the sign flips of its code's two low bits.
//
// `shift8` = 8 * (columns by which this lane's steps begin early, 0..63): the lane's step covers
// columns kc - shift .. kc - shift + 63 (the decompression kernel lets every row's steps end on
// line boundaries of the row's destination; the product passes 0).
template <int ASYM, class AfterWait>
__device__ __forceinline__ void ring_decode_step(RingDecoder &d, lp_u32 table, uint32_t n_groups, uint32_t n_order, int kc,
                                                 uint32_t shift8, AfterWait &&after_wait)
{
    const uint32_t lim8 = 8u * (uint32_t)(kc + kMmAhead) - shift8, end8 = 8u * (uint32_t)(kc + kMmKc) - shift8;
    bool first = true;
    do {
        // Slide the window by one piece where its first piece is used up (once per step as a
        // rule).  The other lanes fetch the piece they already wait for again, so that the
        // load is unconditional and stays in flight until the next slide.
        {
            const bool s8 = d.ci - d.wbase >= 8u;
            if (s8) ring_store_piece(d, 2u * (d.wbase & 8u), d.fut);
            d.wbase += s8 ? 8u : 0u;
            d.pp += s8 ? d.pstr : (uintptr_t)0;
            d.fut = ring_piece_at(d, d.pp + 2u * d.pstr);
        }
        if (first) {
            first = false;
            after_wait();
        }
        // (a loop with its test at the end: with the test in front the compiler keeps two copies of the
        // decoder's state and moves all of it from one to the other every round)
        if (__any(d.left != 0u && d.pos8 < end8 && d.ci - d.wbase <= 12u)) do {
            const bool go = d.left != 0u && d.pos8 <= lim8 && d.ci - d.wbase <= 12u;
            // The entry this round applies; a lane that sits out applies an empty one, which stores
            // three zeros at the column where its next run starts: nothing was written there yet, and
            // it is never a column of the step being completed (kMmAhead keeps a lane's position below
            // kc + 128), so the loop body has no branch and the stores need not be waited for.
            const uint32_t e0 = go ? d.ent : 0u;
            // move on to codeword ci + go: its entry is the one read a round ago (go) or still e0,
            // the code after it c2 (go) or still c1; this round's reads go out before anything else
            const uint32_t csel = go ? d.c2 : d.c1;
            d.ent = go ? (d.ent_n ^ d.flips_n) : d.ent;
            d.ci += go ? 1u : 0u;
            d.ent_n = table[ring_entry_index(csel, n_groups, n_order)];
            d.flips_n = order_flips(csel);
            d.c1 = csel;
            d.c2 = ring_code_at(d, d.ci + 2u);
            __builtin_amdgcn_sched_barrier(0);  // the round's two reads go out before the rest of its work
#pragma unroll
            for (int z = 0; z < kRunMaxNonzeros; z++) {
                const uint32_t t = d.pos8 + ((e0 >> (8 + 8 * z)) & 0xFFu);  // 8 * column + the field's low three bits
                const uint32_t col = (t >> 3) & (uint32_t)(kMmRing - 1);
                // value bits of the field (2: +1, 6: -1): as they are (asymmetric grid: byte selectors), or
                // at the top of the byte (0x40 / 0xC0; the store keeps the low eight bits)
                *(lw_u8)(uintptr_t)(d.wrow + col) = (unsigned char)(ASYM ? (t & 6u) : (t << 5));
            }
            d.pos8 += e0 & 0xFFu;
            d.left -= go ? 1u : 0u;
        } while (__any(d.left != 0u && d.pos8 < end8 && d.ci - d.wbase <= 12u));
    } while (__any(d.left != 0u && d.pos8 < end8));
}

// The half of the ring that held step c becomes columns kc + 128 .. kc + 191: cleared after
// the step's reads.
__device__ __forceinline__ void ring_clear_half(const RingDecoder &d, int c)
{
#pragma unroll
    for (int i = 0; i < kMmKc / 8; i++) ((lw_u64)(uintptr_t)(d.wrow + (uint32_t)((c & 1) * kMmKc)))[i] = 0ull;
}

// ---- the matrix-core product ----
//
// Every wavefront works on its own: its 64 lanes decode 64 consecutive rows into their rings,
// and when all of them have passed the next 64 columns the wavefront multiplies those 64 x 64
// weights with the tile's activations, which every lane fetches straight from global memory
// in the layout the matrix cores want (a token's 8 consecutive columns = one 16-byte load;
// the eight wavefronts of a workgroup read the same lines, which the caches serve).  No
// workgroup barrier inside an item.
//
// MB: blocks of 16 tokens in the tile (1, 2 or 4).  D[token][row] += X[token][k] * W^T[k][row]
// with v_mfma_f32_16x16x32_bf16: operand lane l holds 8 consecutive k (group l / 16) of token
// or row l % 16; accumulator v of lane l is token 4 * (l / 16) + v, row l % 16 of the block.
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int MB, int EPI, int ASYM>
__device__ __forceinline__ void mm_item(const ProductArgs &a, const qmoe_matrix &M, int rblk, int slot0, int ntok,
                                        lp_u32 table, uint32_t wt, uint32_t win)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lg = lane >> 4;

    // The second product writes to the tokens' own rows of the output, scaled by their gates.  Lane t asks
    // for token t's row and gate now, among the other trips to memory of the set-up (two registers for the
    // length of the item); the lanes swap them when the results are written.
    int tok_own = 0;
    float gate_own = 1.0f;
    if constexpr (EPI == 0) {
        const int t = min(lane, ntok - 1);
        tok_own = a.perm ? a.perm[slot0 + t] : slot0 + t;
    }

    // ---- this lane's row (the wavefront's 64 rows are block `rblk` of the matrix) and its codewords
    const int r0 = rblk * 64;
    const int row = r0 + lane;
    const bool row_live = row < a.rows;
    RingDecoder dec;
    ring_setup(dec, M, row, row_live, wt + (uint32_t)(tid * kMmWRowBytes), win + (uint32_t)(tid * kMmWinBytes));
    if constexpr (EPI == 0) gate_own = a.gate ? a.gate[tok_own] : 1.0f;

    // ---- this lane's part of the activations: token 16 * mb + l16, columns 8 * lg .. 8 * lg + 7 of every 32
    uintptr_t xsrc[MB];
    uint32_t xmul[MB];  // bytes from one column's value to the next column's, in units of 2: 1, or (tiled) the block's tokens
    bool x_ok[MB];
    const bool x_col = 8 * lg + 8 <= a.cols;
#pragma unroll
    for (int mb = 0; mb < MB; mb++) {
        const int t = 16 * mb + l16;
        x_ok[mb] = t < ntok;
        xmul[mb] = 1u;
        // (a lane whose columns do not exist -- fewer than 8 * lg + 8 columns -- reads column 0 and drops it;
        // a lane without a token reads the block's first token, or row 0)
        const size_t col0 = x_col ? 8 * (size_t)lg : (size_t)0;
        if (a.x_tiled) {
            const int tb = min(16, ntok - 16 * mb);  // tokens in this block (<= 0: no such block)
            const size_t block0 = tb > 0 ? (size_t)(slot0 + 16 * mb) : (size_t)slot0;
            const size_t j = x_ok[mb] ? (size_t)l16 : (size_t)0;
            xmul[mb] = (uint32_t)max(tb, 1);
            xsrc[mb] = reinterpret_cast<uintptr_t>(a.x) + 2 * (block0 * (size_t)a.ldx + col0 * (size_t)xmul[mb] + 8 * j);
        } else {
            size_t xrow = 0;
            if (x_ok[mb]) {
                const int tok = a.perm ? a.perm[slot0 + t] : slot0 + t;
                xrow = a.x_by_slot ? (size_t)(slot0 + t) : (size_t)tok;
            }
            xsrc[mb] = reinterpret_cast<uintptr_t>(a.x) + 2 * (xrow * (size_t)a.ldx + col0);
        }
        x_ok[mb] = x_ok[mb] && x_col;
    }
    // Loads are unconditional (a lane without a token, or past the last column, reads a valid
    // address -- column 8 * lg of some row -- and drops the value): a load under a branch would
    // be waited for at the end of the branch instead of staying in flight.
    const int x_last = x_col ? a.cols - 8 * lg - 8 : 0;  // last column offset this lane may read at
    auto load_x = [&](int mb, int k) -> u32x4 {
        return *(gp_u32x4)(xsrc[mb] + 2 * (uintptr_t)xmul[mb] * (uintptr_t)min(k, x_last));
    };
    auto keep_x = [&](int mb, const u32x4 &v, int k) -> u32x4 {
        return (x_ok[mb] && k <= x_last) ? v : u32x4{0u, 0u, 0u, 0u};
    };

    f32x4 acc[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; mb++)
#pragma unroll
        for (int nb = 0; nb < 4; nb++) acc[mb][nb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // asymmetric grid: the grid points of the four rows whose weights this lane feeds to the matrix cores
    uint32_t g_hi[4] = {0u, 0u, 0u, 0u}, g_lo[4] = {0u, 0u, 0u, 0u};
    if constexpr (ASYM) {
#pragma unroll
        for (int nb = 0; nb < 4; nb++) {
            const int rl = 16 * nb + l16;
            uint32_t pair = 0u;  // a row past the end, or a matrix without a pair array, multiplies as zeros
            if (r0 + rl < a.rows && M.minmax_bf16) pair = ((gp_u32)M.minmax_bf16)[r0 + rl];
            g_hi[nb] = pair << 16;
            g_lo[nb] = pair & 0xFFFF0000u;
        }
    }
    const uint32_t wfrag = wt + (uint32_t)((64 * wave + l16) * kMmWRowBytes + 8 * lg);
    const int nsteps = (a.cols + kMmKc - 1) / kMmKc;
    const uint32_t n_groups = (uint32_t)a.n_groups, n_order = (uint32_t)a.n_order;

    ring_prime(dec, table, n_groups, n_order);

    u32x4 xa[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; mb++)
#pragma unroll
        for (int ks = 0; ks < 2; ks++) xa[mb][ks] = keep_x(mb, load_x(mb, 32 * ks), 32 * ks);

    for (int c = 0; c < nsteps; c++) {
        const int kc = c * kMmKc;
        // ---- decode until every lane has passed column kc + 64; the next step's activations are
        // fetched right after the window's wait, a whole step ahead
        u32x4 xn[MB][2];
        ring_decode_step<ASYM>(dec, table, n_groups, n_order, kc, 0u, [&]() {
            int k_next = kc + kMmKc;
            asm volatile("" : "+s"(k_next));
#pragma unroll
            for (int mb = 0; mb < MB; mb++)
#pragma unroll
                for (int ks = 0; ks < 2; ks++) xn[mb][ks] = load_x(mb, k_next + 32 * ks);
        });
        // the rows this wavefront multiplies are the ones its own lanes wrote
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- multiply step c
        const uint32_t wf = wfrag + (uint32_t)((c & 1) * kMmKc);
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            bf16x8 bw[4], ax[MB];
#pragma unroll
            for (int nb = 0; nb < 4; nb++) {
                const unsigned long long d = *(lp_u64)(uintptr_t)(wf + (uint32_t)(nb * 16 * kMmWRowBytes + 32 * ks));
                if constexpr (ASYM)
                    bw[nb] = mm_expand_minmax((uint32_t)d, (uint32_t)(d >> 32), g_hi[nb], g_lo[nb]);
                else
                    bw[nb] = mm_expand((uint32_t)d, (uint32_t)(d >> 32));
            }
#pragma unroll
            for (int mb = 0; mb < MB; mb++) __builtin_memcpy(&ax[mb], &xa[mb][ks], 16);
#pragma unroll
            for (int mb = 0; mb < MB; mb++)
#pragma unroll
                for (int nb = 0; nb < 4; nb++)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ax[mb], bw[nb], acc[mb][nb], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        ring_clear_half(dec, c);
#pragma unroll
        for (int mb = 0; mb < MB; mb++)
#pragma unroll
            for (int ks = 0; ks < 2; ks++) xa[mb][ks] = keep_x(mb, xn[mb][ks], kc + kMmKc + 32 * ks);
    }

    // accumulator v of lane l: token 16 * mb + 4 * (l / 16) + v, row 16 * nb + l % 16 of the wavefront's 64
    // (second product: output row and gate of each of the lane's tokens, from the lane that holds them)
    int tok_of[MB][4];
    float gate_of[MB][4];
    if constexpr (EPI == 0) {
#pragma unroll
        for (int mb = 0; mb < MB; mb++)
#pragma unroll
            for (int v = 0; v < 4; v++) {
                const int t = 16 * mb + 4 * lg + v;  // < 64
                tok_of[mb][v] = __shfl(tok_own, t, 64);
                gate_of[mb][v] = __shfl(gate_own, t, 64);
            }
    }
#pragma unroll
    for (int nb = 0; nb < 4; nb++) {
        const int r = r0 + 16 * nb + l16;
        if (r < a.rows) {
            // symmetric grid: the weights were +-2; asymmetric: they were the grid points themselves
            const float scale = ASYM ? 1.0f : 0.5f * half_bits_to_float(((gp_u16)M.scale_f16)[r]);
#pragma unroll
            for (int mb = 0; mb < MB; mb++) {
#pragma unroll
                for (int v = 0; v < 4; v++) {
                    const int t = 16 * mb + 4 * lg + v;
                    if (t < ntok) {
                        const float val = acc[mb][nb][v] * scale;
                        if constexpr (EPI == 0) {
                            reinterpret_cast<float *>(a.out)[(size_t)tok_of[mb][v] * a.ld_out + r] = gate_of[mb][v] * val;
                        } else {
                            const float h = val > 0.0f ? val : 0.0f;
                            size_t at = (size_t)(slot0 + t) * a.ld_out + r;
                            if (a.out_tiled) {
                                const int tb = min(16, ntok - 16 * mb);
                                at = (size_t)(slot0 + 16 * mb) * a.ld_out + ((size_t)(r >> 3) * tb + (4 * lg + v)) * 8 + (r & 7);
                            }
                            reinterpret_cast<uint16_t *>(a.out)[at] = float_to_bf16_bits(h);
                        }
                    }
                }
            }
        }
    }
}

template <int EPI, int ASYM>
__global__ __launch_bounds__(kMmThreads) void k_product_mm(const ProductArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const size_t table_bytes = ((size_t)a.n_order * 4 + 15) & ~(size_t)15;
    uint32_t *table_w = reinterpret_cast<uint32_t *>(smem);
    unsigned char *wt = smem + table_bytes;                           // [512][kMmWRowBytes] rings
    unsigned char *win = wt + (size_t)kMmThreads * kMmWRowBytes;      // [512][kMmWinBytes] codeword windows

    // A unit of work is 64 rows of one (expert, token tile) item, and a wavefront takes it alone: after
    // the table is staged the wavefronts of a workgroup share nothing and meet at no barrier, so one
    // wavefront's set-up (a chain of trips to memory) runs under the others' arithmetic, a matrix
    // whose rows are no multiple of 512 leaves no wavefront idle, and the units are small enough to
    // pack well.  A layer call brings a list of items and a device counter that hands the units out;
    // the single-matrix call has neither: its items are the tiles of 64 consecutive tokens of
    // `single`, its units dealt out round robin.
    const bool listed = a.items != nullptr;
    const int n_items = listed ? min(*a.n_items_dev, a.max_items) : (a.batch + kMmTokens - 1) / kMmTokens;
    const int total = (int)min((long long)n_items * a.mm_row_blocks, 0x7FFFFFFFLL);
    const int wave = (int)threadIdx.x >> 6, lane = (int)threadIdx.x & 63, waves = kMmThreads / 64;
    // No more workgroups than fill all their wavefronts stay (a workgroup holds its compute unit's LDS whole,
    // so one that runs half empty keeps the other kernels of a layer call off that compute unit); the
    // single-matrix call, which is after latency, spreads its units over as many compute units as it can.
    if (total <= 0 || (int)blockIdx.x >= (listed ? (total + waves - 1) / waves : total)) return;
    int *next_base = reinterpret_cast<int *>(win + (size_t)kMmThreads * kMmWinBytes);  // [1], in-step hand-out only
    int *tok_sums = next_base + 1;                                                      // [2]
    if (threadIdx.x < 2) tok_sums[threadIdx.x] = 0;
    stage_words(table_w, a.order_table, a.n_order);
    __syncthreads();
    // In step or each wavefront for itself (see the loop)?  In step when most of the tokens sit in tiles of
    // more than 32: those read 4-8 KB of activations per wavefront and step.
    bool in_step = false;
    if (listed && a.mm_in_step) {
        int big = 0, all = 0;
        for (int i = threadIdx.x; i < n_items; i += kMmThreads) {
            const int n = max(0, min(a.items[i].ntok, kMmTokens));
            all += n;
            big += n > 32 ? n : 0;
        }
        if (all) {
            atomicAdd(&tok_sums[0], all);
            atomicAdd(&tok_sums[1], big);
        }
        __syncthreads();
        in_step = 2 * tok_sums[1] > tok_sums[0];
    }

    const uint32_t wt_addr = (uint32_t)(uintptr_t)(lw_u8)wt, win_addr = (uint32_t)(uintptr_t)(lw_u8)win;
    // (round robin over the workgroups first, then over their wavefronts: few units spread over many compute units)
    int g_static = wave * (int)gridDim.x + (int)blockIdx.x;
    for (;;) {
        int g = g_static;
        if (in_step) {
            // The wavefronts of a workgroup take eight consecutive units together and start them together:
            // where the activations are not stored by token blocks (the first product of a layer) their
            // operand loads touch a line per token, and eight wavefronts that ask for the same lines at the
            // same time are served by one fetch.  (Measured both ways: a layer with few, crowded experts is
            // 3 % faster in step, one with many experts of 8-32 tokens 7 % faster without.)
            __syncthreads();
            if (threadIdx.x == 0) *next_base = atomicAdd(a.work_counter, waves);
            __syncthreads();
            const int base = *next_base;
            if (base >= total) break;
            g = base + wave;
            if (g >= total) continue;
        } else if (listed) {
            int got = 0;
            if (lane == 0) got = atomicAdd(a.work_counter, 1);
            g = __builtin_amdgcn_readfirstlane(got);
        }
        g_static += (int)gridDim.x * waves;
        if (g >= total) break;
        const int idx = g / a.mm_row_blocks;
        const int rblk = g - idx * a.mm_row_blocks;
        Item it;
        if (listed) {
            it = a.items[idx];
        } else {
            it.expert = 0;
            it.slot0 = idx * kMmTokens;
            it.ntok = a.batch - idx * kMmTokens;
        }
        const int expert = it.expert, slot0 = it.slot0;
        const int ntok = min(it.ntok, kMmTokens);
        if (expert < 0 || expert >= a.n_experts || ntok < 1) continue;
        const qmoe_matrix M = a.mats ? a.mats[expert] : a.single;
        if (ntok <= 16)
            mm_item<1, EPI, ASYM>(a, M, rblk, slot0, ntok, (lp_u32)table_w, wt_addr, win_addr);
        else if (ntok <= 32)
            mm_item<2, EPI, ASYM>(a, M, rblk, slot0, ntok, (lp_u32)table_w, wt_addr, win_addr);
        else
            mm_item<4, EPI, ASYM>(a, M, rblk, slot0, ntok, (lp_u32)table_w, wt_addr, win_addr);
    }
}

// ---------------------------------------------------------------- decompression of whole matrices
//
// The codec without the product: dense ternary (int8) or scaled bf16 copies of compressed
// matrices, for consumers that want a plain matrix (a library GEMM, a check).  The ring
// decoder of the matrix-core product: a workgroup of 512 lanes owns up to 512 rows, one lane
// per row; after each 64-column step a wavefront writes out the 64 x 64 tile its own lanes
// decoded, 8 rows per store instruction with 8 lanes covering a row's 64 columns, so that
// the stores are whole 64- or 128-byte runs.  Wavefronts never wait for each other.

// OUT 0: int8 in {-1, 0, +1}; 1: bf16(scale of the row) with the weight's sign, or 0;
// 2: the row's bf16 grid point w_max or w_min, or 0 (asymmetric grid)
template <int OUT>
__global__ __launch_bounds__(kMmThreads) void k_decompress(const DecompressArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const size_t table_bytes = ((size_t)a.n_order * 4 + 15) & ~(size_t)15;
    uint32_t *table_w = reinterpret_cast<uint32_t *>(smem);
    stage_words(table_w, a.order_table, a.n_order);
    __syncthreads();
    lp_u32 table = (lp_u32)table_w;
    const uint32_t wt = (uint32_t)(uintptr_t)(lw_u8)(smem + table_bytes);               // [512][kMmWRowBytes] rings
    const uint32_t win = wt + (uint32_t)(kMmThreads * kMmWRowBytes);                     // [512][kMmWinBytes] codeword windows
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = lane & 7, sub_row = lane >> 3;  // write-out role: columns 8*seg.., rows sub_row + 8*i
    const uint32_t n_groups = (uint32_t)a.n_groups, n_order = (uint32_t)a.n_order;
    // A row's 64-column steps begin early by as many columns as it takes for their ends to fall on
    // 128-byte (bf16) or 64-byte (int8) boundaries of the row's destination: a matrix whose rows are no
    // multiple of that long would otherwise have every run of every other row straddle two lines.
    // (Destinations are 16-byte aligned and cols is a multiple of 8, so a shift is a multiple of 8 columns.)
    constexpr int kBpe = OUT == 0 ? 1 : 2, kRunBytes = kMmKc * kBpe;
    const bool shifted = ((size_t)a.cols * kBpe) % kRunBytes != 0;
    const int nsteps = (a.cols + kMmKc - 1) / kMmKc + (shifted ? 1 : 0);

    // Which matrices have a destination: one bit each, so that the workgroups share the matrices that
    // are asked for evenly (dealt out over all matrices, a workgroup's share of those would be a matter of luck).
    using lw_mask = __attribute__((address_space(3))) unsigned long long *;
    lw_mask mask = (lw_mask)(uintptr_t)(win + (uint32_t)(kMmThreads * kMmWinBytes));  // [(n_mats + 63) / 64]
    const int mask_words = (a.n_mats + 63) / 64;
    for (int w = wave; w < mask_words; w += kMmThreads / 64) {
        const int m = 64 * w + lane;
        const unsigned long long bits = __ballot(m < a.n_mats && a.out[m] != nullptr);
        if (lane == 0) mask[w] = bits;
    }
    __syncthreads();
    long long n_wanted = 0;
    for (int w = 0; w < mask_words; w++) n_wanted += __popcll(mask[w]);
    const long long total = n_wanted * a.row_blocks;

    for (long long g = blockIdx.x; g < total; g += gridDim.x) {
        const int nth = (int)(g / a.row_blocks);  // which of the wanted matrices
        const int blk = (int)(g - (long long)nth * a.row_blocks);
        int m;
        {
            int w = 0, rem = nth;
            for (;; w++) {
                const int n = __popcll(mask[w]);
                if (rem < n) break;
                rem -= n;
            }
            unsigned long long bits = mask[w];
            for (int i = 0; i < rem; i++) bits &= bits - 1ull;
            // (the same in every lane; said so, the matrix descriptor is read into scalar registers)
            m = __builtin_amdgcn_readfirstlane(64 * w + (int)__ffsll((long long)bits) - 1);
        }
        // (a pointer read from memory is a generic one to the compiler; stores through it would go out as
        // generic-address stores, which count as LDS traffic too and make every wait of the decoder a full one)
        const uintptr_t out = reinterpret_cast<uintptr_t>(a.out[m]);
        // columns by which row r's steps begin early
        auto row_shift = [&](int r) -> int {
            const int lead = (int)((out + (uintptr_t)kBpe * (uintptr_t)r * (uintptr_t)a.cols) % kRunBytes);  // bytes past a boundary
            return lead / kBpe;  // = (64 - columns up to the row's first boundary) mod 64
        };
        const qmoe_matrix M = a.mats[m];
        const int r0 = blk * a.rows_per_block;
        const int row = r0 + tid;
        const bool row_live = tid < a.rows_per_block && row < a.rows;
        RingDecoder dec;
        ring_setup(dec, M, row, row_live, wt + (uint32_t)(tid * kMmWRowBytes), win + (uint32_t)(tid * kMmWinBytes));

        // the eight rows this lane writes out: which of them exist, and their bf16 scale in both
        // halves of a register (OUT 2: the (w_min, w_max) pair as stored, w_min in the low half)
        bool r_ok[8];
        uint32_t s2[8];
        int sh[8];  // the shifts of those rows
        const uint32_t shift8 = shifted && row_live ? 8u * (uint32_t)row_shift(row) : 0u;  // this lane's own row
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int rl = 64 * wave + sub_row + 8 * i;
            r_ok[i] = rl < a.rows_per_block && r0 + rl < a.rows;
            sh[i] = shifted && r_ok[i] ? row_shift(r0 + rl) : 0;
            // (loads without a branch, from row r0 where there is no row: the eight are in flight together)
            const int rr = r_ok[i] ? r0 + rl : min(r0, a.rows - 1);
            s2[i] = 0u;
            if constexpr (OUT == 2) {
                if (M.minmax_bf16) {
                    const uint32_t pair = ((gp_u32)M.minmax_bf16)[rr];
                    s2[i] = r_ok[i] ? pair : 0u;
                }
            }
            if constexpr (OUT == 1) {
                const uint32_t b = float_to_bf16_bits(half_bits_to_float(((gp_u16)M.scale_f16)[rr]));
                s2[i] = r_ok[i] ? (b | (b << 16)) : 0u;
            }
        }
        ring_prime(dec, table, n_groups, n_order);

        for (int c = 0; c < nsteps; c++) {
            const int kc = c * kMmKc;
            ring_decode_step<OUT == 2>(dec, table, n_groups, n_order, kc, shift8, []() {});
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // the eight reads first (every lane reads, from inside the workgroup's rings), then the stores
            unsigned long long d[8];
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const int rl = 64 * wave + sub_row + 8 * i;
                const uint32_t ring_col = (uint32_t)(kc - sh[i] + 8 * seg) & (uint32_t)(kMmRing - 1);  // 8-aligned: no wrap inside
                d[i] = *(lp_u64)(uintptr_t)(wt + (uint32_t)(rl * kMmWRowBytes) + ring_col);
            }
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const int r = r0 + 64 * wave + sub_row + 8 * i;
                const int k = kc - sh[i] + 8 * seg;
                if (r_ok[i] && k >= 0 && k + 8 <= a.cols) {
                    const uint32_t w0 = (uint32_t)d[i], w1 = (uint32_t)(d[i] >> 32);
                    const size_t at = (size_t)r * a.cols + k;
                    if constexpr (OUT == 0) {
                        // ring byte 0x40 -> 0x01, 0xC0 -> 0xFF, 0 -> 0
                        const uint32_t o0 = ((w0 >> 6) & 0x01010101u) | (((w0 >> 7) & 0x01010101u) * 0xFEu);
                        const uint32_t o1 = ((w1 >> 6) & 0x01010101u) | (((w1 >> 7) & 0x01010101u) * 0xFEu);
                        *(gw_u64)(out + at) = (unsigned long long)o0 | ((unsigned long long)o1 << 32);
                    } else if constexpr (OUT == 2) {
                        const bf16x8 v = mm_expand_minmax(w0, w1, s2[i] << 16, s2[i] & 0xFFFF0000u);
                        u32x4 o;
                        __builtin_memcpy(&o, &v, 16);
                        *(gw_u32x4)(out + 2 * at) = o;
                    } else {
                        u32x4 o;
#pragma unroll
                        for (int h = 0; h < 4; h++) {
                            // two ring bytes -> the high bytes of two 16-bit halves: 0x4000 / 0xC000 / 0
                            const uint32_t e = __builtin_amdgcn_perm(0u, h < 2 ? w0 : w1, (h & 1) ? 0x030c020cu : 0x010c000cu);
                            const uint32_t present = ((e >> 14) & 0x00010001u) * 0xFFFFu;
                            o[h] = ((e & 0x80008000u) | s2[i]) & present;
                        }
                        *(gw_u32x4)(out + 2 * at) = o;
                    }
                }
            }
            // the 64 columns of this lane's ring that held its step are cleared for the step after next:
            // after the reads above
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int j = 0; j < kMmKc / 8; j++) {
                const uint32_t ring_col = ((uint32_t)(8 * kc + 64 * j) - shift8) >> 3 & (uint32_t)(kMmRing - 1);
                *(lw_u64)(uintptr_t)(dec.wrow + ring_col) = 0ull;
            }
        }
    }
}

}  // namespace

size_t mm_lds_bytes(int n_order)
{
    return (((size_t)n_order * 4 + 15) & ~(size_t)15) + (size_t)kMmThreads * kMmWRowBytes +
           (size_t)kMmThreads * kMmWinBytes + 16;
}

size_t decompress_lds_bytes(int n_order, int n_mats)
{
    return (((size_t)n_order * 4 + 15) & ~(size_t)15) + (size_t)kMmThreads * kMmWRowBytes +
           (size_t)kMmThreads * kMmWinBytes + 8 * (((size_t)n_mats + 63) / 64);
}

void mm_rows(int rows, int *row_blocks, int *rows_per_block)
{
    const int nb = (rows + kMmThreads - 1) / kMmThreads;
    const int per = (rows + nb - 1) / nb;
    *row_blocks = nb;
    *rows_per_block = std::min(kMmThreads, (per + 63) / 64 * 64);
}

qmoe_status launch_product_mm(ProductArgs a, const MmPlan &mp, hipStream_t s)
{
    a.mm_row_blocks = (a.rows + 63) / 64;  // units of 64 rows, one wavefront each
    auto launch = [&](auto kernel) -> qmoe_status {
        const qmoe_status st = allow_lds(kernel, mp.smem);
        if (st != QMOE_OK) return st;
        hipLaunchKernelGGL(kernel, dim3(mp.grid), dim3(kMmThreads), mp.smem, s, a);
        return QMOE_OK;
    };
    qmoe_status st;
    if (a.minmax)
        st = a.epilogue ? launch(k_product_mm<1, 1>) : launch(k_product_mm<0, 1>);
    else
        st = a.epilogue ? launch(k_product_mm<1, 0>) : launch(k_product_mm<0, 0>);
    if (st != QMOE_OK) return st;
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}


qmoe_status launch_decompress(const DecompressArgs &a, int out_kind, bool minmax, int grid, size_t smem, hipStream_t s)
{
    qmoe_status st;
    if (out_kind == 0) {
        if ((st = allow_lds(k_decompress<0>, smem)) != QMOE_OK) return st;
        hipLaunchKernelGGL(k_decompress<0>, dim3(grid), dim3(kMmThreads), smem, s, a);
    } else if (minmax) {
        if ((st = allow_lds(k_decompress<2>, smem)) != QMOE_OK) return st;
        hipLaunchKernelGGL(k_decompress<2>, dim3(grid), dim3(kMmThreads), smem, s, a);
    } else {
        if ((st = allow_lds(k_decompress<1>, smem)) != QMOE_OK) return st;
        hipLaunchKernelGGL(k_decompress<1>, dim3(grid), dim3(kMmThreads), smem, s, a);
    }
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

}  // namespace qmoe
