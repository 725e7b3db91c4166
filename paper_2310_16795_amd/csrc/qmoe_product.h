// The fused decode + product kernel (Section 4.3.3 of the paper defines what is computed;
// the mapping below is this library's own), included by the translation units that
// instantiate it (one per grid: {-s, 0, +s} and {w_min, 0, w_max}).
//
//  - Lane per row range: the rows of a matrix are dealt evenly over all lanes of the
//    workgroups that share a pass; a lane's rows are consecutive, so its codewords are one
//    contiguous piece of the stream, which it decodes sequentially -- the running column
//    index is a scalar per lane, exactly the paper's sequential decoder, 64 of them per
//    wavefront.  No prefix sum across lanes, no reduction, no idle lanes at row ends.
//  - A codeword is looked up in a compact "run entry" table in LDS (length plus up to three
//    signed non-zero positions), so the arithmetic per codeword is three gathers from the
//    activations in LDS, not 28 multiply-adds.
//  - The activations of a tile of one, two or four (eight) tokens sit in LDS as bf16, so one
//    decoded weight is applied to all tokens of the tile with one LDS read.
//  - Workgroups are persistent and fetch (expert, token tile, row block) items, which the
//    dispatch kernel listed, from a device counter; experts without tokens never appear.
#pragma once

#include "qmoe_dev.h"

namespace qmoe {
namespace {

// Per-lane decoder state for one item.
template <int TBI, int ASYM = 0>
struct LaneState {
    float acc[TBI * (1 + ASYM)];  // running sums since the last row that was written (ASYM: see accumulate)
    uint32_t pos8;     // 8 * (column reached in the current row)
    int row, rb;       // current row, end of this lane's rows
    uint32_t sraw;     // one-token tiles: the current row's scale (or grid pair) as stored, read when the row began
};

// What a lane needs to write a finished row; everything it reads sits in LDS, so
// that closing a row never waits on global memory (which would also wait for the
// stream and table prefetches in flight).
struct RowSink {
    lp_u16 scale_s;   // binary16 scales of the block's rows (asymmetric grid: bf16 (w_min, w_max) pairs, 4 bytes a row)
    int r0;           // first row of the block
    const __attribute__((address_space(3))) int *tok_ids;   // output token of each tile slot
    const __attribute__((address_space(3))) float *gate_s;  // gate of each tile slot
    int ntok, slot0;
    float acc_unit;   // what one unit of a running sum stands for: 1, or 0.5 where the weights were applied as +-2
    uint32_t out_s;   // LDS byte address of the block's staged results [tile][out_rows] (bf16 or fp32), 0 = none
    int out_rows;     // rows of the block
    float gate0;      // gate of tile slot 0
};

// the scale (binary16) or grid pair (two bf16) of the block's row i, as stored
template <int ASYM>
__device__ __forceinline__ uint32_t row_scale_raw(const RowSink &rs, int i)
{
    if constexpr (ASYM) return ((lp_u32)rs.scale_s)[i];
    else return (uint32_t)rs.scale_s[i];
}

template <int TBI, int EPI, int ASYM = 0>
__device__ __forceinline__ void write_row(const ProductArgs &a, const LaneState<TBI, ASYM> &st,
                                          const float (&sum)[TBI * (1 + ASYM)], const RowSink &rs)
{
    float scale = 0.0f, mid = 0.0f;  // y = scale * (signed sum) + mid * (sum under |weight|)
    if constexpr (ASYM) {
        const uint32_t pair = ((lp_u32)rs.scale_s)[st.row - rs.r0];
        const float w_min = __uint_as_float(pair << 16), w_max = __uint_as_float(pair & 0xFFFF0000u);
        scale = 0.5f * (w_max - w_min);
        mid = 0.5f * (w_max + w_min);
    } else {
        scale = half_bits_to_float(rs.scale_s[st.row - rs.r0]);
    }
    scale *= rs.acc_unit;  // exact: a power of two
    mid *= rs.acc_unit;
#pragma unroll
    for (int t = 0; t < TBI; t++) {
        if (t < rs.ntok) {
            float v = sum[t] * scale;
            if constexpr (ASYM) v = fmaf(sum[TBI + t], mid, v);
            if constexpr (EPI == 0) {
                if (rs.out_s) {
                    *(__attribute__((address_space(3))) float *)(uintptr_t)(
                        rs.out_s + 4u * (uint32_t)(t * rs.out_rows + (st.row - rs.r0))) = rs.gate_s[t] * v;
                } else {
                    const int tok = rs.tok_ids[t];
                    reinterpret_cast<float *>(a.out)[(size_t)tok * a.ld_out + st.row] = rs.gate_s[t] * v;
                }
            } else {
                const float h = v > 0.0f ? v : 0.0f;
                if (rs.out_s) {
                    // a pass's hidden values leave the compute unit as whole lines at its end
                    // (one 2-byte store per lane and row would reach HBM as partial lines)
                    *(__attribute__((address_space(3))) uint16_t *)(uintptr_t)(
                        rs.out_s + 2u * (uint32_t)(t * rs.out_rows + (st.row - rs.r0))) = float_to_bf16_bits(h);
                } else {
                    reinterpret_cast<uint16_t *>(a.out)[(size_t)(rs.slot0 + t) * a.ld_out + st.row] =
                        float_to_bf16_bits(h);
                }
            }
        }
    }
}

// General form: one decoded entry at a time, the row closed as soon as it is full.
// Works for any width and any table; used for narrow matrices (several row ends may
// fall into eight codewords) and for tables without run entries.
template <int TBI, int DICT, int EPI, int ASYM>
__device__ __forceinline__ void consume1(const ProductArgs &a, LaneState<TBI, ASYM> &st, const Entry &e,
                                         uint32_t cols8, uint32_t xs_addr, const RowSink &rs)
{
    accumulate<TBI, DICT, ASYM>(e, xs_addr, st.pos8, st.acc);
    st.pos8 += 8u * (uint32_t)entry_len<DICT>(e);
    if (__any(st.pos8 >= cols8)) {
        if (st.pos8 >= cols8) {
            if (st.row < st.rb) write_row<TBI, EPI, ASYM>(a, st, st.acc, rs);
#pragma unroll
            for (int t = 0; t < TBI * (1 + ASYM); t++) st.acc[t] = 0.0f;
            st.pos8 -= cols8;
            st.row += 1;
            if constexpr (TBI == 1) st.sraw = row_scale_raw<ASYM>(rs, min(st.row, st.rb) - rs.r0);
        }
    }
}

// One token, the block's results staged in LDS: write the lane's current row from the sums
// `snap`.  The row's scale was read when the row began, so nothing here waits on a read.
template <int EPI, int ASYM>
__device__ __forceinline__ void stage_row_one(const LaneState<1, ASYM> &st, const float (&snap)[1 + ASYM], const RowSink &rs)
{
    float v;
    if constexpr (ASYM) {
        const float w_min = __uint_as_float(st.sraw << 16), w_max = __uint_as_float(st.sraw & 0xFFFF0000u);
        v = fmaf(snap[1], 0.5f * (w_max + w_min), snap[0] * (0.5f * (w_max - w_min)));
    } else {
        v = snap[0] * half_bits_to_float((uint16_t)st.sraw);
    }
    const uint32_t i = (uint32_t)(st.row - rs.r0);
    if constexpr (EPI == 0) {
        *(__attribute__((address_space(3))) float *)(uintptr_t)(rs.out_s + 4u * i) = rs.gate0 * v;
    } else {
        *(__attribute__((address_space(3))) uint16_t *)(uintptr_t)(rs.out_s + 2u * i) =
            float_to_bf16_bits(v > 0.0f ? v : 0.0f);
    }
}

// Fast form for run tables and rows of more than 224 values (at most one row end per
// eight codewords): the eight entries are applied without a branch in between, so
// their LDS gathers overlap; the running sum is never reset inside, a row end only
// records the sum reached (`snap`), and the row is written once after the eight.
// One token: the activations are 8-byte records {0, +x, 0, -x} and an entry's field
// is the byte offset of the wanted 16-bit slot from the record of the run's first
// column (unused fields land on a zero), so a non-zero costs one add.
template <int TBI, int DICT, int EPI, int ASYM>
__device__ __forceinline__ void consume8(const ProductArgs &a, LaneState<TBI, ASYM> &st, const Entry (&e)[8],
                                         uint32_t cols8, uint32_t xs_addr, const RowSink &rs)
{
    constexpr int NA = TBI * (1 + ASYM);
    // Where each of the eight runs begins, as 8 * column.  Past the row's end the position
    // falls back by the row's width: p - cols8 wraps around to a huge number for every p
    // below cols8, so the smaller of the two is the position either way.  Eight runs span
    // at most 8 * 28 columns < cols, so the position after the eight is below the one
    // before them exactly when a row ended among them, and a run ended its row exactly when
    // the next one begins before it.  (Empty entries, which stand for slots that are not
    // the lane's, move nothing.)
    uint32_t pos[9];
    uint32_t p = st.pos8;
#pragma unroll
    for (int j = 0; j < 8; j++) {
        pos[j] = p;
        p += e[j].e0 & 0xFFu;
        p = min(p, p - cols8);
    }
    pos[8] = p;
    const bool wrapped = p < st.pos8;
    st.pos8 = p;
    float part[8][NA];  // the sums after each of the eight
    if constexpr (TBI == 1) {
        // the three bf16 values of a codeword are added with two packed dot products
        // against (1, 1): two of them share a register, no widening shifts
        uint32_t x[24];
        uint32_t xa[ASYM ? 24 : 1];  // asymmetric grid: the same inputs with their own sign (+x of each record)
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const uint32_t rec = pos[j];  // the activations begin at LDS address 0 (the caller checks)
#pragma unroll
            for (int z = 0; z < 3; z++) {
                const uint32_t addr = rec + ((e[j].e0 >> (8 + 8 * z)) & 0xFFu);
                x[3 * j + z] = (uint32_t)(*(lp_u16)(uintptr_t)addr);
                // the -x slot is 4 bytes after the +x slot; an unused field stays on the zero slot
                if constexpr (ASYM) xa[3 * j + z] = (uint32_t)(*(lp_u16)(uintptr_t)(addr & ~4u));
            }
        }
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const uint32_t one2 = 0x3F803F80u;
        bf16x2 ones;
        __builtin_memcpy(&ones, &one2, 4);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const uint32_t pair = x[3 * j] | (x[3 * j + 1] << 16);
            bf16x2 p2, p1;
            __builtin_memcpy(&p2, &pair, 4);
            __builtin_memcpy(&p1, &x[3 * j + 2], 4);
            st.acc[0] = __builtin_amdgcn_fdot2_f32_bf16(p2, ones, st.acc[0], false);
            st.acc[0] = __builtin_amdgcn_fdot2_f32_bf16(p1, ones, st.acc[0], false);
            part[j][0] = st.acc[0];
            if constexpr (ASYM) {
                const uint32_t pair_a = xa[3 * j] | (xa[3 * j + 1] << 16);
                bf16x2 a2, a1;
                __builtin_memcpy(&a2, &pair_a, 4);
                __builtin_memcpy(&a1, &xa[3 * j + 2], 4);
                st.acc[NA - 1] = __builtin_amdgcn_fdot2_f32_bf16(a2, ones, st.acc[NA - 1], false);
                st.acc[NA - 1] = __builtin_amdgcn_fdot2_f32_bf16(a1, ones, st.acc[NA - 1], false);
                part[j][NA - 1] = st.acc[NA - 1];
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            if constexpr (DICT != kDictWords) accumulate_tile<TBI, ASYM>(e[j].e0, xs_addr, pos[j], st.acc);
            else accumulate<TBI, DICT, ASYM>(e[j], xs_addr, pos[j], st.acc);
#pragma unroll
            for (int t = 0; t < NA; t++) part[j][t] = st.acc[t];
        }
    }
    if (__any(wrapped)) {
        if (wrapped) {
            float snap[NA];
#pragma unroll
            for (int t = 0; t < NA; t++) snap[t] = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const bool ended = pos[j + 1] < pos[j];
#pragma unroll
                for (int t = 0; t < NA; t++) snap[t] = ended ? part[j][t] : snap[t];
            }
#pragma unroll
            for (int t = 0; t < NA; t++) st.acc[t] -= snap[t];
            if (st.row < st.rb) {
                if constexpr (TBI == 1) {
                    if (rs.out_s) stage_row_one<EPI, ASYM>(st, snap, rs);
                    else write_row<TBI, EPI, ASYM>(a, st, snap, rs);
                } else {
                    write_row<TBI, EPI, ASYM>(a, st, snap, rs);
                }
            }
            st.row += 1;
            // the next row's scale is asked for now and not needed before that row ends
            if constexpr (TBI == 1) st.sraw = row_scale_raw<ASYM>(rs, min(st.row, st.rb) - rs.r0);
        }
    }
}

// table entries of the eight codewords held in one 16-byte piece of the stream
template <int DICT>
__device__ __forceinline__ void lookup8(const ProductArgs &a, const u32x4 &v, lp_u32 lds_run, Entry (&e)[8])
{
    if constexpr (DICT == kDictOrder || DICT == kDictOrderL2) {
        const uint32_t n_groups3 = 3u * (uint32_t)a.n_groups, last = (uint32_t)a.n_order - 1u;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            e[2 * j].e1 = 0u; e[2 * j + 1].e1 = 0u;
            if constexpr (DICT == kDictOrder) order_entry2(lds_run, v[j], n_groups3, last, e[2 * j].e0, e[2 * j + 1].e0);
            else order_entry2((gp_u32)a.order_table, v[j], n_groups3, last, e[2 * j].e0, e[2 * j + 1].e0);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            e[2 * j] = lookup_entry<DICT>(a, v[j] & 0xFFFFu, lds_run);
            e[2 * j + 1] = lookup_entry<DICT>(a, v[j] >> 16, lds_run);
        }
    }
}

// One block of one (expert, token tile) item: every lane decodes its own rows.
//
// The rows of the matrix are dealt out evenly over all lanes of the workgroups that
// share the item; a lane's rows are consecutive, so its codewords are one contiguous
// piece of the stream, which it reads in aligned 16-byte pieces (eight codewords, two
// pieces in flight ahead of the one being applied) and decodes sequentially:
// no prefix sum across lanes, no reduction -- the running column index is a scalar
// per lane, exactly the paper's sequential decoder, 64 of them per wavefront.  Table
// entries are fetched eight codewords ahead of their use.
template <int TBI, int DICT, int EPI, int ASYM>
__device__ __forceinline__ void product_block(const ProductArgs &a, const qmoe_matrix &M, int blk,
                                              uint32_t xs_addr, const RowSink &rs_in, lp_u32 lds_run)
{
    const bool fast = DICT != kDictWords && a.cols > 224 && (TBI != 1 || xs_addr == 0u);
    RowSink rs = rs_in;
    // token tiles on the fast form apply the weights as +-2 (see accumulate_tile)
    rs.acc_unit = (fast && TBI != 1) ? 0.5f : 1.0f;
    const int nlanes = (int)blockDim.x * a.blocks_per_pass;
    const int gl = blk * (int)blockDim.x + (int)threadIdx.x;
    const int base_rows = a.rows / nlanes, extra = a.rows - base_rows * nlanes;
    const int ra = gl * base_rows + min(gl, extra);
    const int rb = ra + base_rows + (gl < extra ? 1 : 0);
    gp_u32 row_off = (gp_u32)M.row_off;
    uint32_t K0 = 0, K1 = 0;
    if (ra < rb) {
        const uint32_t cap = min(M.n_codes, kMaxCodes);
        K1 = min(row_off[rb], cap);
        K0 = min(row_off[ra], K1);
    }
    const uint32_t n = K1 - K0;  // codewords of this lane
    // The stream is read in aligned 16-byte pieces (eight codewords); `rel` is the stream
    // index (relative to K0) of the first slot of the lane's first piece.
    // (a lane without codewords reads the matrix's first piece, never past the stream's end)
    // Rows back to back: a lane's pieces follow each other.  Lane-interleaved layout (built for
    // exactly this launch's lanes per matrix): the lane's stream starts on a piece of its own
    // and piece p sits 64 p pieces further on, next to the same piece of the wavefront's other
    // lanes, so that the wavefront's 64 loads are one run of 1 KiB.
    const bool interleaved = M.lanes != 0u;
    if (interleaved && M.lanes != (uint32_t)nlanes) return;  // not the launch the layout was built for
    uintptr_t first_byte = reinterpret_cast<uintptr_t>(M.codes) + (n ? 2 * (uintptr_t)K0 : (uintptr_t)0);
    if (interleaved && n)
        first_byte = reinterpret_cast<uintptr_t>(M.codes) +
                     16u * ((uintptr_t)((gp_u32)M.wave_off)[gl >> 6] + (uintptr_t)(gl & 63));
    const uint32_t lead = (uint32_t)(first_byte & 15u);
    const uintptr_t chunk = first_byte - lead;
    const uintptr_t pstride = interleaved ? 1024u : 16u;  // from a piece of the lane to its next
    const int rel = -(int)(lead >> 1);
    const int my_pieces = n ? (int)((lead + 2u * n + 15u) >> 4) : 0;
    int npieces = my_pieces;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) npieces = max(npieces, __shfl_xor(npieces, d, 64));

    const uint32_t cols8 = 8u * (uint32_t)a.cols;
    LaneState<TBI, ASYM> st;
#pragma unroll
    for (int t = 0; t < TBI * (1 + ASYM); t++) st.acc[t] = 0.0f;
    st.pos8 = 0;
    st.row = ra;
    st.rb = rb;
    st.sraw = 0u;
    if constexpr (TBI == 1) st.sraw = row_scale_raw<ASYM>(rs, min(ra, rb) - rs.r0);

    // Piece p + 2 is being loaded and the entries of piece p + 1 looked up while piece p
    // is applied.
    const uintptr_t last_piece = chunk + pstride * (uintptr_t)max(my_pieces - 1, 0);
    auto load_piece = [&](int p) -> u32x4 {
        // lanes past their own end re-read their last piece (its slots are masked out below)
        const uintptr_t at = chunk + pstride * (uintptr_t)p;
        return *(gp_u32x4)(at < last_piece ? at : last_piece);
    };
    auto apply = [&](Entry (&e)[8], int r) {
        // r: stream index (relative to K0) of the piece's first slot
        const bool whole = r >= 0 && (uint32_t)r + 8u <= n;  // all eight are this lane's codewords
        if (fast) {
            // Slots that are not this lane's codewords (before its first, after its last, and
            // everything once the lane is done while others in the wavefront are not) become
            // empty entries: no columns, no non-zeros.  The wavefront stays on the branch-free
            // form from its first piece to its last.
            if (!__all(whole)) {
#pragma unroll
                for (int j = 0; j < 8; j++)
                    if ((uint32_t)(r + j) >= n) e[j].e0 = 0u;
            }
            consume8<TBI, DICT, EPI, ASYM>(a, st, e, cols8, xs_addr, rs);
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++) {
                Entry ej = e[j];
                if ((uint32_t)(r + j) >= n) { ej.e0 = 0u; ej.e1 = 0u; }  // not this lane's codeword
                consume1<TBI, DICT, EPI, ASYM>(a, st, ej, cols8, xs_addr, rs);
            }
        }
    };
    Entry ea[8], eb[8];
    // Issue priorities that take turns: of the three wavefronts that share a SIMD (workgroups
    // of 768 lanes), one runs the first piece of a pair at high priority and the second
    // at low, one the other way round, one stays in the middle.  The wavefronts of a SIMD then
    // sit in different stretches of the loop (vector arithmetic only / throttled by the LDS
    // queue) more of the time: 2 % on the c2048 layer, measured; fixed priorities, or three
    // that rotate, gain nothing.
    const int turn = ((int)threadIdx.x >> 8) % 3;
    if (turn == 2) __builtin_amdgcn_s_setprio(1);
    // Four pieces (64 bytes of a lane's stream) are asked for together and stay in flight for
    // a whole loop round, so that a 128-byte line is visited twice or three times instead of
    // eight times, a round apart each time (the lanes of a workgroup keep more lines in use
    // than the first-level cache holds, so every visit is a request to L2).
    // (One-token tiles only: with the registers of a token tile on top, the pieces in flight
    // would spill.)
    if constexpr (TBI != 1) {
        u32x4 cb = load_piece(1);
        lookup8<DICT>(a, load_piece(0), lds_run, ea);
        for (int p = 0; p < npieces; p += 2) {
            if (turn == 0) __builtin_amdgcn_s_setprio(2);
            else if (turn == 1) __builtin_amdgcn_s_setprio(0);
            const u32x4 cc = load_piece(p + 2);
            lookup8<DICT>(a, cb, lds_run, eb);
            apply(ea, rel + 8 * p);
            if (turn == 0) __builtin_amdgcn_s_setprio(0);
            else if (turn == 1) __builtin_amdgcn_s_setprio(2);
            cb = load_piece(p + 3);
            lookup8<DICT>(a, cc, lds_run, ea);
            apply(eb, rel + 8 * p + 8);
        }
        __builtin_amdgcn_s_setprio(0);
        return;
    }
    u32x4 q0 = load_piece(0), q1 = load_piece(1), q2 = load_piece(2), q3 = load_piece(3);
    lookup8<DICT>(a, q0, lds_run, ea);
    for (int p = 0; p < npieces; p += 4) {
        const u32x4 n0 = load_piece(p + 4), n1 = load_piece(p + 5), n2 = load_piece(p + 6), n3 = load_piece(p + 7);
        if (turn == 0) __builtin_amdgcn_s_setprio(2);
        else if (turn == 1) __builtin_amdgcn_s_setprio(0);
        lookup8<DICT>(a, q1, lds_run, eb);
        apply(ea, rel + 8 * p);
        if (turn == 0) __builtin_amdgcn_s_setprio(0);
        else if (turn == 1) __builtin_amdgcn_s_setprio(2);
        lookup8<DICT>(a, q2, lds_run, ea);
        apply(eb, rel + 8 * p + 8);
        if (turn == 0) __builtin_amdgcn_s_setprio(2);
        else if (turn == 1) __builtin_amdgcn_s_setprio(0);
        lookup8<DICT>(a, q3, lds_run, eb);
        apply(ea, rel + 8 * p + 16);
        if (turn == 0) __builtin_amdgcn_s_setprio(0);
        else if (turn == 1) __builtin_amdgcn_s_setprio(2);
        lookup8<DICT>(a, n0, lds_run, ea);
        apply(eb, rel + 8 * p + 24);
        q1 = n1; q2 = n2; q3 = n3;
    }
    __builtin_amdgcn_s_setprio(0);
}

// ---------------------------------------------------------------- fused decode + product

// EPI 0: fp32 out[token][r] = gate * s_r * acc      (second product, and the plain matvec)
// EPI 1: bf16 out[slot][r]  = relu(s_r * acc)        (first product, writes the hidden vector)
// LDS: activations | token ids | leading run entries.  Activations are bf16, for one
// token as 8-byte records {0, +x, 0, -x} per column, for 2/4/8 tokens packed per column.
// ASYM: rows on the grid {w_min, 0, w_max} (bf16 pair per row) instead of {-s, 0, +s}.
// At most kProductMaxThreads lanes per workgroup: three wavefronts per SIMD, which leaves
// each of them 168 vector registers (a bound of 1024 would cap them at 128).
template <int DICT, int EPI, int ASYM>
__global__ __launch_bounds__(kProductMaxThreads) void k_product(const ProductArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *xs_w = reinterpret_cast<uint16_t *>(smem);
    const size_t xs_bytes = (size_t)(a.cols + kPadCols) * max(a.tb_max, 4) * sizeof(uint16_t);
    int *tok_ids = reinterpret_cast<int *>(smem + xs_bytes);            // [kMaxTokenTile] output token
    int *x_rows = tok_ids + kMaxTokenTile;                              // [kMaxTokenTile] input row
    float *gate_s = reinterpret_cast<float *>(x_rows + kMaxTokenTile);  // [kMaxTokenTile] gate
    int *next_item = reinterpret_cast<int *>(gate_s + kMaxTokenTile);   // [1]
    uint16_t *scale_w = reinterpret_cast<uint16_t *>(smem + xs_bytes + 128);  // [rows_per_item] row scales
    const size_t scale_bytes = ((size_t)a.rows_per_item * (ASYM ? 4 : 2) + 15) / 16 * 16;
    uint32_t *lds_run_w = reinterpret_cast<uint32_t *>(smem + xs_bytes + 128 + scale_bytes);
    const size_t table_entries = DICT == kDictOrder ? (size_t)a.n_order : (DICT == kDictRunLds ? (size_t)a.lds_dict_entries : 0);
    uint16_t *out_w = reinterpret_cast<uint16_t *>(smem + xs_bytes + 128 + scale_bytes + ((table_entries * 4 + 15) & ~(size_t)15));
    lp_u16 xs = (lp_u16)xs_w;
    lp_u32 lds_run = (lp_u32)lds_run_w;
    const uint32_t xs_addr = (uint32_t)(uintptr_t)xs;  // LDS byte address of the activations

    int n_pass;
    if (a.items) {
        n_pass = min(*a.n_items_dev, a.max_items);
    } else {
        n_pass = (a.batch + a.tb_max - 1) / a.tb_max;
    }
    const int total = (int)min((long long)n_pass * a.blocks_per_pass, 0x7FFFFFFFLL);
    // Items are handed out one at a time from a device counter when there is one (uneven
    // experts balance themselves), otherwise each workgroup takes an equal contiguous share.
    const int per = (total + (int)gridDim.x - 1) / (int)gridDim.x;
    int g_static = per * (int)blockIdx.x;
    const int g_static_end = min(total, g_static + per);
    if (total <= 0 || (!a.work_counter && g_static >= g_static_end)) return;

    if constexpr (DICT == kDictRunLds) {
        stage_words(lds_run_w, a.run, a.lds_dict_entries);
    } else if constexpr (DICT == kDictOrder) {
        stage_words(lds_run_w, a.order_table, a.n_order);
    }

    int cur_pass = -1, ntok = 0, slot0 = 0, expert = 0, tbi = 1;
    for (;;) {
        __syncthreads();  // everyone is done with the previous item (activations, token ids, next_item)
        if (threadIdx.x == 0) {
            int g;
            if (a.work_counter) {
                g = atomicAdd(a.work_counter, 1);
                if (g >= total) g = -1;
            } else {
                g = g_static < g_static_end ? g_static : -1;
            }
            *next_item = g;
        }
        g_static++;
        __syncthreads();
        const int g = *next_item;
        if (g < 0) break;
        const int pass = g / a.blocks_per_pass;
        const int blk = g - pass * a.blocks_per_pass;
        if (pass != cur_pass) {
            if (a.items) {
                const Item it = a.items[pass];
                expert = it.expert; slot0 = it.slot0; ntok = it.ntok;
            } else {
                expert = 0; slot0 = pass * a.tb_max; ntok = min(a.tb_max, a.batch - slot0);
            }
            if (expert < 0 || expert >= a.n_experts || ntok < 1) ntok = 0;
            ntok = min(ntok, a.tb_max);
            tbi = ntok <= 1 ? 1 : (ntok <= 2 ? 2 : (ntok <= 4 ? 4 : 8));
            if (threadIdx.x < kMaxTokenTile) {
                const int t = threadIdx.x;
                int tok = 0, xr = 0;
                if (t < ntok) {
                    tok = a.perm ? a.perm[slot0 + t] : slot0 + t;
                    xr = a.x_by_slot ? slot0 + t : tok;
                }
                tok_ids[t] = tok;
                x_rows[t] = xr;
                gate_s[t] = (a.gate && t < ntok) ? a.gate[tok] : 1.0f;
            }
            __syncthreads();
            auto row_of = [&](int t) { return x_rows[t]; };
            switch (tbi) {
            case 1: stage_x_one(xs_w, a.x + (size_t)x_rows[0] * a.ldx, a.cols, ntok > 0, true); break;
            case 2: stage_x_tile<4>(xs_w, a.x, row_of, ntok, a.ldx, a.cols); break;  // eight bytes per column as well
            case 4: stage_x_tile<4>(xs_w, a.x, row_of, ntok, a.ldx, a.cols); break;
            default: stage_x_tile<8>(xs_w, a.x, row_of, ntok, a.ldx, a.cols); break;
            }
            __syncthreads();
            cur_pass = pass;
        }
        if (ntok == 0) continue;
        const qmoe_matrix M = a.mats ? a.mats[expert] : a.single;
        // the block's rows: lanes blk*T .. blk*T+T-1 of the even split (see product_block)
        const int nlanes = (int)blockDim.x * a.blocks_per_pass;
        const int base_rows = a.rows / nlanes, extra = a.rows - base_rows * nlanes;
        const int gl0 = blk * (int)blockDim.x, gl1 = gl0 + (int)blockDim.x;
        const int r0 = gl0 * base_rows + min(gl0, extra);
        const int r1 = min(gl1 * base_rows + min(gl1, extra), r0 + a.rows_per_item);
        if constexpr (ASYM) {
            // a matrix without a pair array decodes to zeros
            for (int i = threadIdx.x; i < r1 - r0; i += blockDim.x)
                reinterpret_cast<uint32_t *>(scale_w)[i] = M.minmax_bf16 ? ((gp_u32)M.minmax_bf16)[r0 + i] : 0u;
        } else {
            for (int i = threadIdx.x; i < r1 - r0; i += blockDim.x) scale_w[i] = ((gp_u16)M.scale_f16)[r0 + i];
        }
        __syncthreads();
        RowSink rs;
        rs.scale_s = (lp_u16)scale_w;
        rs.r0 = r0;
        rs.tok_ids = (const __attribute__((address_space(3))) int *)tok_ids;
        rs.gate_s = (const __attribute__((address_space(3))) float *)gate_s;
        rs.ntok = ntok;
        rs.slot0 = slot0;
        const bool staged = a.stage_out && (r0 % 8) == 0;
        rs.out_s = staged ? (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)out_w : 0u;
        rs.out_rows = (r1 - r0 + 7) & ~7;
        rs.gate0 = gate_s[0];
        rs.acc_unit = 1.0f;
        switch (tbi) {
        case 1: product_block<1, DICT, EPI, ASYM>(a, M, blk, xs_addr, rs, lds_run); break;
        case 2: product_block<2, DICT, EPI, ASYM>(a, M, blk, xs_addr, rs, lds_run); break;
        case 4: product_block<4, DICT, EPI, ASYM>(a, M, blk, xs_addr, rs, lds_run); break;
        default: product_block<8, DICT, EPI, ASYM>(a, M, blk, xs_addr, rs, lds_run); break;
        }
        if (staged) {
            // the block's results, staged in LDS, go out as whole 16-byte pieces
            __syncthreads();
            constexpr int kPer = EPI == 1 ? 8 : 4;  // values per piece
            using value_t = typename std::conditional<EPI == 1, uint16_t, float>::type;
            const int nrows = r1 - r0, per_tok = rs.out_rows / kPer;
            const value_t *stage = reinterpret_cast<const value_t *>(out_w);
            value_t *out = reinterpret_cast<value_t *>(a.out);
            for (int i = threadIdx.x; i < ntok * per_tok; i += blockDim.x) {
                const int t = i / per_tok, j = i - t * per_tok;
                const size_t out_row = EPI == 1 ? (size_t)(slot0 + t) : (size_t)tok_ids[t];
                const value_t *src = stage + (size_t)t * rs.out_rows + kPer * j;
                value_t *dst = out + out_row * a.ld_out + r0 + kPer * j;
                if (kPer * j + kPer <= nrows) {
                    *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
                } else {
                    for (int k = 0; kPer * j + k < nrows; k++) dst[k] = src[k];
                }
            }
        }
    }
}


template <int DICT, int EPI, int ASYM>
qmoe_status launch_product_grid(const ProductArgs &a, const ProductPlan &p, hipStream_t s)
{
    const qmoe_status st = allow_lds(k_product<DICT, EPI, ASYM>, p.smem);
    if (st != QMOE_OK) return st;
    hipLaunchKernelGGL((k_product<DICT, EPI, ASYM>), dim3(p.grid), dim3(p.threads), p.smem, s, a);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

// The kernel that reads the table where the plan put it, for grid ASYM.
template <int ASYM>
qmoe_status launch_product_for(const ProductArgs &a, const ProductPlan &p, bool run, hipStream_t s)
{
    if (a.code_order && p.order_l2)
        return a.epilogue ? launch_product_grid<kDictOrderL2, 1, ASYM>(a, p, s) : launch_product_grid<kDictOrderL2, 0, ASYM>(a, p, s);
    if (a.code_order)
        return a.epilogue ? launch_product_grid<kDictOrder, 1, ASYM>(a, p, s) : launch_product_grid<kDictOrder, 0, ASYM>(a, p, s);
    if (!run) return a.epilogue ? launch_product_grid<kDictWords, 1, ASYM>(a, p, s) : launch_product_grid<kDictWords, 0, ASYM>(a, p, s);
    if (p.lds_dict_entries > 0)
        return a.epilogue ? launch_product_grid<kDictRunLds, 1, ASYM>(a, p, s) : launch_product_grid<kDictRunLds, 0, ASYM>(a, p, s);
    return a.epilogue ? launch_product_grid<kDictRun, 1, ASYM>(a, p, s) : launch_product_grid<kDictRun, 0, ASYM>(a, p, s);
}

}  // namespace
}  // namespace qmoe
