// HIP kernels for gfx950 (CDNA4, wave64) and their launch code.
//
// Work decomposition of the fused decode + product kernel (Section 4.3.3 of the
// paper defines what is computed; the mapping below is this library's own):
//  - a 16-lane DPP row ("group") owns a contiguous range of matrix rows and with
//    it one contiguous piece of the codeword stream; each lane takes one codeword
//    per step, so a step covers 16 consecutive codewords = 32 contiguous bytes,
//    four groups per wavefront, codewords fetched two steps ahead of their use;
//  - the running column index of the paper's sequential decoder becomes an
//    inclusive prefix sum of the run lengths inside the group (four DPP row
//    shifts), with the previous step's total carried in through lane 0; a row is
//    complete when the sum reaches `cols`, and the group then reduces and writes it;
//  - a codeword is looked up in a compact "run entry" table (length plus up to
//    three signed non-zero positions), so the arithmetic per codeword is three
//    gathers from the activations in LDS, not 28 multiply-adds;
//  - the activations of up to eight tokens sit interleaved in LDS as bf16, so one
//    decoded weight is applied to all tokens of the tile with one LDS read;
//  - workgroups are persistent and walk a list of (expert, token tile, row
//    block) items that the dispatch kernel wrote; experts without tokens never
//    appear in it.
#include <hip/hip_runtime.h>
#include <cmath>
#include <mutex>
#include <type_traits>

#include <atomic>
#include <cstdio>

#include "qmoe_internal.h"

namespace qmoe {
namespace {

std::atomic<int> g_last_hip_error{0};

inline bool hip_failed(hipError_t e)
{
    if (e == hipSuccess) return false;
    g_last_hip_error.store((int)e);
    return true;
}
#define QMOE_HIP_TRY(expr)                           \
    do {                                             \
        if (hip_failed(expr)) return QMOE_E_HIP;     \
    } while (0)

constexpr int kPadCols = 32;     // zeroed activations past the last column (a run is at most 28 long)
constexpr int kMaxTokenTile = 8;
constexpr int kMaxCols = 32768;
constexpr int kMaxExperts = 16384;
constexpr int kMaxTokens = 1 << 20;
constexpr int kMaxRowsPerItem = 1024;
constexpr uint32_t kMaxCodes = 0xFFFFFF00u;  // keeps `kb += 16` from wrapping
constexpr int kLayerCounters = 16;

struct Item {  // one (expert, token tile) unit of work; row blocks are enumerated on the fly
    int expert, slot0, ntok, pad;
};

struct ProductArgs {
    const qmoe_matrix *mats;  // device array indexed by expert, or nullptr -> `single`
    qmoe_matrix single;
    const uint32_t *run;      // run-entry table, 65536 entries
    const uint32_t *words;    // interchange-layout table, 65536 x 2
    const Item *items;        // device list, or nullptr -> tiles of `batch` tokens of matrix 0
    const int *n_items_dev;   // device count (with items), clamped to max_items
    int max_items;
    int n_experts;
    int batch;
    const int *perm;          // slot -> token, or nullptr (identity)
    const uint16_t *x;        // bf16 activations, row stride ldx
    int x_by_slot;            // 1: row = slot, 0: row = token
    int ldx;
    void *out;
    int ld_out;
    const float *gate;        // by token, or nullptr
    int epilogue;             // 0: fp32 out[token][r] = gate*s*acc   1: bf16 out[slot][r] = relu(s*acc)
    int rows, cols;
    int rows_per_item, blocks_per_pass;
    int tb_max;
    int lds_dict_entries;     // leading run entries copied to LDS (0 = none)
    int stage_out;            // first product: results of a block staged in LDS and written as whole lines (LDS after the table)
    int *work_counter;        // device counter (zeroed by the dispatch kernel) for handing out items, or nullptr
    const uint32_t *order_table;  // device-order table (n_order entries, the first n_groups are groups)
    int n_groups, n_order;
    int code_order;           // numbering of the streams (decode_dense only; the product picks its kernel)
    int mm_row_blocks, mm_rows_per_block;  // matrix-core kernel: workgroups per matrix, rows each takes (<= 512)
    int mm_stagger;           // matrix-core kernel: the two wavefronts of a SIMD half a step apart
    int minmax;               // rows on the grid {w_min, 0, w_max} (host side: which kernel to launch)
};

// ---------------------------------------------------------------- device helpers

template <int CTRL>
__device__ __forceinline__ int dpp0(int v)  // lanes without a source get 0
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118, kRowRor1 = 0x121;

// inclusive prefix sum over the 16 lanes of a DPP row
__device__ __forceinline__ int row_scan16(int v)
{
    v += dpp0<kRowShr1>(v);
    v += dpp0<kRowShr2>(v);
    v += dpp0<kRowShr4>(v);
    v += dpp0<kRowShr8>(v);
    return v;
}

// sum over the 16 lanes of a DPP row, result valid in lane 15 of the row
__device__ __forceinline__ float row_sum16_to_last(float v)
{
    v += __int_as_float(dpp0<kRowShr8>(__float_as_int(v)));
    v += __int_as_float(dpp0<kRowShr4>(__float_as_int(v)));
    v += __int_as_float(dpp0<kRowShr2>(__float_as_int(v)));
    v += __int_as_float(dpp0<kRowShr1>(__float_as_int(v)));
    return v;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)  // round to nearest even, finite or inf
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    _Float16 f;
    __builtin_memcpy(&f, &h, sizeof f);
    return (float)f;
}

// Global-memory pointers with their address space spelled out: pointers that reach
// a kernel through memory would otherwise be generic and cost flat loads.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
using gp_u16 = const __attribute__((address_space(1))) uint16_t *;
using gp_u32 = const __attribute__((address_space(1))) uint32_t *;
using gp_u64 = const __attribute__((address_space(1))) unsigned long long *;
using gp_u32x4 = const __attribute__((address_space(1))) u32x4 *;
using lp_u32 = const __attribute__((address_space(3))) uint32_t *;
using lp_u16 = const __attribute__((address_space(3))) uint16_t *;

// Copy n 32-bit words from global memory to LDS with the whole workgroup (both 16-byte
// aligned): 16 bytes per lane and up to eight loads in flight per lane before the first
// store.  (A plain word-by-word loop waits for every load before it issues the next; for the
// 65 KB table that was 20-60 us at the start of every workgroup.)
__device__ __forceinline__ void stage_words(uint32_t *dst_lds, const uint32_t *src, int n)
{
    const int n4 = n >> 2;  // whole 16-byte pieces
    gp_u32x4 s4 = (gp_u32x4)src;
    u32x4 *d4 = reinterpret_cast<u32x4 *>(dst_lds);
    const int step = (int)blockDim.x;
    for (int i0 = (int)threadIdx.x; i0 < n4; i0 += 8 * step) {
        u32x4 v[8];
#pragma unroll
        for (int k = 0; k < 8; k++) v[k] = s4[min(i0 + k * step, n4 - 1)];
#pragma unroll
        for (int k = 0; k < 8; k++)
            if (i0 + k * step < n4) d4[i0 + k * step] = v[k];
    }
    for (int i = 4 * n4 + (int)threadIdx.x; i < n; i += step) dst_lds[i] = ((gp_u32)src)[i];
}

// ---- activations of a tile into LDS (whole workgroup).  The loads of eight columns (one
// token) or of all the tile's tokens (tiles) are issued before the first store: a loop that
// loads and stores one value at a time waits for every load in turn.
//
// One token: 8-byte records {0, +x, 0, -x} (with_neg) or {0, x, 0, 0}; columns cols ..
// cols + kPadCols - 1, and everything when `live` is false, are zero records.
__device__ __forceinline__ void stage_x_one(uint16_t *xs_w, const uint16_t *xrow, int cols, bool live, bool with_neg)
{
    const int n = cols + kPadCols, step = (int)blockDim.x;
    gp_u16 x = (gp_u16)xrow;
    for (int c0 = (int)threadIdx.x; c0 < n; c0 += 8 * step) {
        uint32_t v[8];
#pragma unroll
        for (int k = 0; k < 8; k++) v[k] = x[min(c0 + k * step, cols - 1)];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const int c = c0 + k * step;
            if (c < n) {
                const bool in = live && c < cols;
                const uint32_t pos = in ? v[k] : 0u, neg = (in && with_neg) ? (v[k] ^ 0x8000u) : 0u;
                reinterpret_cast<uint2 *>(xs_w)[c] = make_uint2(pos << 16, neg << 16);
            }
        }
    }
}

// TBI tokens (2, 4, 8): bf16 [column][TBI]; token t of the tile is row x_rows[t] of x (tokens
// from ntok on are zeros).  x_rows holds at least one valid row.
template <int TBI, typename RowOf>
__device__ __forceinline__ void stage_x_tile(uint16_t *xs_w, const uint16_t *xbase, RowOf row_of, int ntok, int ldx,
                                             int cols)
{
    const int n = cols + kPadCols, step = (int)blockDim.x;
    gp_u16 x = (gp_u16)xbase;
    size_t off[TBI];
#pragma unroll
    for (int t = 0; t < TBI; t++) off[t] = (size_t)row_of(min(t, ntok - 1)) * (size_t)ldx;
    for (int c = (int)threadIdx.x; c < n; c += step) {
        const int cc = min(c, cols - 1);
        uint32_t v[TBI];
#pragma unroll
        for (int t = 0; t < TBI; t++) v[t] = x[off[t] + cc];
        uint32_t w[TBI / 2];
#pragma unroll
        for (int t = 0; t < TBI; t += 2) {
            const uint32_t lo = (c < cols && t < ntok) ? v[t] : 0u, hi = (c < cols && t + 1 < ntok) ? v[t + 1] : 0u;
            w[t / 2] = lo | (hi << 16);
        }
        uint32_t *dst = reinterpret_cast<uint32_t *>(xs_w) + (size_t)c * (TBI / 2);
#pragma unroll
        for (int i = 0; i < TBI / 2; i++) dst[i] = w[i];
    }
}

// Entry of a device-order code from the group/single table (see qmoe_internal.h):
// codes below 4 * n_groups share table[code >> 2], the rest are single entries at
// table[code - 3 * n_groups]; the index is the larger of the two expressions (the
// subtraction saturating at zero): they cross exactly at code = 4 * n_groups.  The two low
// bits of every code flip the sign bits of fields 1 and 2; the single entries are stored
// with those flips already applied once, so that the second application restores them
// and no case distinction is needed.
template <typename TablePtr>
__device__ __forceinline__ uint32_t order_entry(TablePtr table, uint32_t code, uint32_t n_groups, uint32_t n_order)
{
    const uint32_t u = max(code >> 2, __builtin_elementwise_sub_sat(code, 3u * n_groups));
    // bit 0 -> bit 18, bit 1 -> bit 26 (two shifts and a mask: a 32-bit multiply runs at a quarter of the rate)
    const uint32_t two = code & 3u;
    const uint32_t flips = ((two << 18) | (two << 25)) & ((1u << 18) | (1u << 26));
    return table[min(u, n_order - 1u)] ^ flips;
}

// The same look-up for the two codewords held in one 32-bit word of the stream.  The
// flip masks of both come out of one packed 16-bit multiply (per half: bit 0 -> bit 2,
// bit 1 -> bit 10, which are bits 18 and 26 of an entry once the half sits on top), and
// the index is the median of the two candidates and the last entry: the larger of the
// two for every code the table knows; for a code it does not know, the last entry or the
// smaller candidate (at most code >> 2 < 16384, inside the space reserved for the table in
// the device blob; in LDS, at worst other bytes of the workgroup's own allocation).
template <typename TablePtr>
__device__ __forceinline__ void order_entry2(TablePtr table, uint32_t w, uint32_t n_groups3, uint32_t last,
                                             uint32_t &e_lo, uint32_t &e_hi)
{
    typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
    const uint32_t two = w & 0x00030003u;
    u16x2 t, k = {0x0204, 0x0204};
    __builtin_memcpy(&t, &two, 4);
    t = t * k;
    uint32_t f;
    __builtin_memcpy(&f, &t, 4);
    const uint32_t c_lo = w & 0xFFFFu, c_hi = w >> 16;
    const uint32_t s_lo = __builtin_elementwise_sub_sat(c_lo, n_groups3);
    const uint32_t s_hi = __builtin_elementwise_sub_sat(c_hi, n_groups3);
    uint32_t i_lo, i_hi;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(i_lo) : "v"(c_lo >> 2), "v"(s_lo), "s"(last));
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(i_hi) : "v"(c_hi >> 2), "v"(s_hi), "s"(last));
    e_lo = table[i_lo] ^ ((f << 16) & 0x04040000u);
    e_hi = table[i_hi] ^ (f & 0x04040000u);
}

// Decode one step (one codeword per lane) and return this lane's run:
// `len` values starting at column `start` (absolute, clamped to cols).
struct Step {
    uint32_t e0, e1;  // run entry (e0) or interchange words (e0,e1)
    int start, len;
};

template <bool RUN>
__device__ __forceinline__ Step decode_step(const ProductArgs &a, const uint16_t *codes, uint32_t k,
                                            uint32_t kend, int l16, int &incl)
{
    Step s;
    s.e0 = 0; s.e1 = 0;
    if (k < kend) {
        const uint32_t code = codes[k];
        if constexpr (RUN) {
            s.e0 = a.code_order ? order_entry((gp_u32)a.order_table, code, (uint32_t)a.n_groups, (uint32_t)a.n_order)
                                : a.run[code];
        } else {
            const uint2 w = reinterpret_cast<const uint2 *>(a.words)[code];
            s.e0 = w.x; s.e1 = w.y;
        }
    }
    s.len = RUN ? (int)((s.e0 & 0xFFu) >> 3) : 2 * (int)(s.e0 & 15u);
    // previous step's total sits in lane 15 of the row; lane 0 takes it in
    const int carry = __builtin_amdgcn_update_dpp(0, incl, kRowRor1, 0xf, 0xf, false);
    incl = row_scan16(s.len + (l16 == 0 ? carry : 0));
    s.start = (int)min((uint32_t)(incl - s.len), (uint32_t)a.cols);  // also catches a wrapped index
    return s;
}

constexpr int kProductMaxThreads = 768;  // largest workgroup of k_product

// where a codeword's entry comes from: run-entry table in L2 | its head in LDS, the rest in L2 |
// interchange words in L2 | device-order table in LDS | device-order table in L2
enum DictMode { kDictRun = 0, kDictRunLds = 1, kDictWords = 2, kDictOrder = 3, kDictOrderL2 = 4 };

struct Entry {
    uint32_t e0, e1;  // run entry (e0), or the two interchange words (e0, e1)
};

// Table look-up without branches, so that the compiler can keep many of them in flight:
// with the head of the run table in LDS, every lane reads LDS and global memory, each
// from entry 0 when the codeword lives in the other one.
template <int DICT>
__device__ __forceinline__ Entry lookup_entry(const ProductArgs &a, uint32_t code, lp_u32 lds_run)
{
    Entry e{0u, 0u};
    if constexpr (DICT == kDictRun) {
        e.e0 = ((gp_u32)a.run)[code];
    } else if constexpr (DICT == kDictRunLds) {
        const bool in_lds = (int)code < a.lds_dict_entries;
        const uint32_t from_lds = lds_run[in_lds ? code : 0u];
        const uint32_t from_l2 = ((gp_u32)a.run)[in_lds ? 0u : code];
        e.e0 = in_lds ? from_lds : from_l2;
    } else if constexpr (DICT == kDictOrder) {
        e.e0 = order_entry(lds_run, code, (uint32_t)a.n_groups, (uint32_t)a.n_order);  // whole table in LDS
    } else if constexpr (DICT == kDictOrderL2) {
        e.e0 = order_entry((gp_u32)a.order_table, code, (uint32_t)a.n_groups, (uint32_t)a.n_order);
    } else {
        const unsigned long long w = ((gp_u64)a.words)[code];
        e.e0 = (uint32_t)w; e.e1 = (uint32_t)(w >> 32);
    }
    return e;
}

template <int DICT>
__device__ __forceinline__ int entry_len(const Entry &e)
{
    return DICT == kDictWords ? 2 * (int)(e.e0 & 15u) : (int)((e.e0 & 0xFFu) >> 3);
}

// activations of one column for the tokens of the tile: bf16 in LDS -> fp32.
// `rec8` is 8 * column.  One token: 8-byte records, +x in the second 16-bit slot;
// 2 / 4 / 8 tokens: packed, 4 / 8 / 16 bytes per column.
template <int TBI>
__device__ __forceinline__ void lds_load_x(uint32_t xs_addr, uint32_t rec8, float (&v)[TBI])
{
    typedef const __attribute__((address_space(3))) uint32_t *p32;
    if constexpr (TBI == 1) {
        v[0] = __uint_as_float((uint32_t)(*(lp_u16)(uintptr_t)(xs_addr + rec8 + 2u)) << 16);
    } else if constexpr (TBI == 2) {
        const uint32_t u = *(p32)(uintptr_t)(xs_addr + (rec8 >> 1));
        v[0] = __uint_as_float(u << 16); v[1] = __uint_as_float(u & 0xFFFF0000u);
    } else if constexpr (TBI == 4) {
        p32 p = (p32)(uintptr_t)(xs_addr + rec8);
        const uint32_t u0 = p[0], u1 = p[1];
        v[0] = __uint_as_float(u0 << 16); v[1] = __uint_as_float(u0 & 0xFFFF0000u);
        v[2] = __uint_as_float(u1 << 16); v[3] = __uint_as_float(u1 & 0xFFFF0000u);
    } else {
        p32 p = (p32)(uintptr_t)(xs_addr + (rec8 << 1));
        const uint32_t u0 = p[0], u1 = p[1], u2 = p[2], u3 = p[3];
        v[0] = __uint_as_float(u0 << 16); v[1] = __uint_as_float(u0 & 0xFFFF0000u);
        v[2] = __uint_as_float(u1 << 16); v[3] = __uint_as_float(u1 & 0xFFFF0000u);
        v[4] = __uint_as_float(u2 << 16); v[5] = __uint_as_float(u2 & 0xFFFF0000u);
        v[6] = __uint_as_float(u3 << 16); v[7] = __uint_as_float(u3 & 0xFFFF0000u);
    }
}

// acc[t] += sum over the entry's non-zeros of weight * x[t][column + position], the
// column given as pos8 = 8 * column.  (The one-token run-table case has its own code
// in consume8; this is the form every other case uses.)
// ASYM (rows on the grid {w_min, 0, w_max}): a second set of sums, acc[TBI + t], takes the
// same inputs with |weight|; the two grid points are applied when the row is written, as
// y = (w_max - w_min)/2 * acc[t] + (w_max + w_min)/2 * acc[TBI + t].
template <int TBI, int DICT, int ASYM = 0>
__device__ __forceinline__ void accumulate(const Entry &e, uint32_t xs_addr, uint32_t pos8,
                                           float (&acc)[TBI * (1 + ASYM)])
{
    if constexpr (DICT != kDictWords) {
#pragma unroll
        for (int j = 0; j < kRunMaxNonzeros; j++) {
            const uint32_t field = (e.e0 >> (8 + 8 * j)) & 0xFFu;
            const int wi = ((int)(e.e0 << (32 - (8 + 8 * j + 3)))) >> 30;  // signed 2-bit weight
            const float w = (float)wi;
            float xv[TBI];
            lds_load_x<TBI>(xs_addr, pos8 + (field & 0xF8u), xv);
#pragma unroll
            for (int t = 0; t < TBI; t++) acc[t] = fmaf(w, xv[t], acc[t]);
            if constexpr (ASYM) {
                const float wa = (float)(wi & 1);
#pragma unroll
                for (int t = 0; t < TBI; t++) acc[TBI + t] = fmaf(wa, xv[t], acc[TBI + t]);
            }
        }
    } else {
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const uint32_t w = h ? e.e1 : e.e0;
            uint32_t m = ((w >> 4) | (w >> 5)) & 0x05555555u;  // bit 2j set <=> symbol j non-zero
            while (m) {
                const int b = __ffs((int)m) - 1;
                m &= m - 1;
                const int sym = (int)((w >> (4 + b)) & 3u);
                const float wt = sym == 2 ? 1.0f : (sym == 1 ? -1.0f : 0.0f);
                float xv[TBI];
                lds_load_x<TBI>(xs_addr, pos8 + 8u * (uint32_t)(14 * h + (b >> 1)), xv);
#pragma unroll
                for (int t = 0; t < TBI; t++) acc[t] = fmaf(wt, xv[t], acc[t]);
                if constexpr (ASYM) {
                    const float wa = sym != 0 ? 1.0f : 0.0f;
#pragma unroll
                    for (int t = 0; t < TBI; t++) acc[TBI + t] = fmaf(wa, xv[t], acc[TBI + t]);
                }
            }
        }
    }
}

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
            accumulate<TBI, DICT, ASYM>(e[j], xs_addr, pos[j], st.acc);
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
                                              uint32_t xs_addr, const RowSink &rs, lp_u32 lds_run)
{
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
    const uintptr_t first_byte = reinterpret_cast<uintptr_t>(M.codes) + 2 * (uintptr_t)K0;
    const uint32_t lead = (uint32_t)(first_byte & 15u);
    const uintptr_t chunk = first_byte - lead;
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
    const uintptr_t last_piece = chunk + 16u * (uintptr_t)max(my_pieces - 1, 0);
    const bool fast = DICT != kDictWords && a.cols > 224 && (TBI != 1 || xs_addr == 0u);
    auto load_piece = [&](int p) -> u32x4 {
        // lanes past their own end re-read their last piece (its slots are masked out below)
        const uintptr_t at = chunk + 16u * (uintptr_t)p;
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
            case 2: stage_x_tile<2>(xs_w, a.x, row_of, ntok, a.ldx, a.cols); break;
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

// ---------------------------------------------------------------- matrix-core product for crowded experts
//
// An expert with many tokens is a dense contraction once its ternary weights are
// in hand: y[token][row] = sum_k x[token][k] * W[row][k].  The scalar kernel above
// would decode the matrix again for every few tokens; this one decodes it once per
// tile of up to 64 tokens.  A workgroup owns up to 512 rows (one lane per row) and
// walks the columns 64 at a time.  Every lane keeps a ring of 128 one-byte columns
// of its row in LDS and decodes its codewords into it sequentially, as far ahead as
// the ring allows (so the lanes of a wavefront, whose codewords end at different
// columns, seldom wait for each other); then each wavefront multiplies the 64
// columns that are complete, for the 64 rows its own lanes decoded, with the
// tokens' activations (staged in LDS, shared by all wavefronts) on the matrix
// cores: D[token][row] += X[token][k] * W^T[k][row], fp32 accumulators in
// registers.  The ring holds the weights as the high byte of bf16 +-2.0 (0x40 /
// 0xC0, low byte zero), expanded to bf16 by a byte permute when a fragment is
// read; the factor 2 is taken out again, exactly, when a row is written.
// Only device-order streams (whole table in LDS) take this path.

constexpr int kMmThreads = 512;
constexpr int kMmKc = 64;                      // columns per step
constexpr int kMmRing = 2 * kMmKc;             // columns a lane's ring holds
constexpr int kMmAhead = kMmRing - 28;         // a codeword may start this far past the step's first column
constexpr int kMmWRowBytes = kMmRing + 8;      // 34 banks per row: 16 consecutive rows read 8 bytes each without conflict
constexpr int kMmXRowBytes = 2 * kMmKc + 16;   // 36 banks per row: 8 consecutive rows read 16 bytes each without conflict
constexpr int kMmTokens = 64;                  // tokens per tile
constexpr int kMmMinTokensDefault = 8;         // experts with fewer tokens stay on the scalar kernel

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

inline size_t mm_lds_bytes(int n_order)
{
    return (((size_t)n_order * 4 + 15) & ~(size_t)15) + (size_t)kMmThreads * kMmWRowBytes +
           2 * (size_t)kMmTokens * kMmXRowBytes + 2 * sizeof(int) * kMmTokens + 16;
}

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

using lw_u8 = __attribute__((address_space(3))) unsigned char *;
using lw_u64 = __attribute__((address_space(3))) unsigned long long *;
using lw_u32x4 = __attribute__((address_space(3))) u32x4 *;
using lp_u64 = const __attribute__((address_space(3))) unsigned long long *;
using lp_u32x4 = const __attribute__((address_space(3))) u32x4 *;
using lp_i32 = const __attribute__((address_space(3))) int *;
using lp_f32 = const __attribute__((address_space(3))) float *;

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also fences global
// memory, which makes every wavefront wait for all its loads in flight: the prefetches
// of codewords and activations would then be exposed at every step.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---- the ring decoder shared by the matrix-core product and the decompression kernel ----
// (macros rather than a struct with member functions: the decoder's state has to stay in
// plain scalar registers, and the compiler keeps it there only when it sees scalars.)
//
// QMOE_RING_ROW_SETUP declares the state for one lane = one row: `left` codewords to go,
// the stream in 16-byte pieces (eight codewords) -- c0..c3 and n0..n3 are the window the
// decoder picks codewords from (index sub = 0..15), `fut` is in flight; pieces past the
// lane's last one re-read the last (never used: `left` runs out first) -- and `pos`, the
// column where the next codeword starts.
#define QMOE_RING_ROW_SETUP(M, row, row_live)                                                           \
    uint32_t left = 0;                                                                                  \
    uintptr_t pp = reinterpret_cast<uintptr_t>((M).codes), last = pp;                                   \
    uint32_t sub = 0;                                                                                   \
    if (row_live) {                                                                                     \
        gp_u32 row_off_ = (gp_u32)(M).row_off;                                                          \
        const uint32_t cap_ = min((M).n_codes, kMaxCodes);                                              \
        const uint32_t K1_ = min(row_off_[(row) + 1], cap_);                                            \
        const uint32_t K0_ = min(row_off_[(row)], K1_);                                                 \
        left = K1_ - K0_;                                                                               \
        const uintptr_t first_byte_ = reinterpret_cast<uintptr_t>((M).codes) + 2 * (uintptr_t)K0_;      \
        const uint32_t lead_ = (uint32_t)(first_byte_ & 15u);                                           \
        pp = first_byte_ - lead_;                                                                       \
        sub = lead_ >> 1;                                                                               \
        last = pp + 16u * (uintptr_t)(left ? ((lead_ + 2u * left + 15u) >> 4) - 1u : 0u);               \
    }                                                                                                   \
    uint32_t c0, c1, c2, c3, n0, n1, n2, n3;                                                            \
    {                                                                                                   \
        const u32x4 a0_ = *(gp_u32x4)pp, a1_ = *(gp_u32x4)(pp + 16u < last ? pp + 16u : last);          \
        c0 = a0_.x; c1 = a0_.y; c2 = a0_.z; c3 = a0_.w;                                                 \
        n0 = a1_.x; n1 = a1_.y; n2 = a1_.z; n3 = a1_.w;                                                 \
    }                                                                                                   \
    u32x4 fut = *(gp_u32x4)(pp + 32u < last ? pp + 32u : last);                                         \
    int pos = 0

// Table entry of the codeword at index `at` (0..15) of the window (anything when at > 15:
// not used then).
#define QMOE_MM_ENTRY_AT(dst, at)                                                                       \
    do {                                                                                                \
        const bool hi8_ = ((at) & 8u) != 0u, hi4_ = ((at) & 4u) != 0u;                                  \
        const uint32_t lo_ = hi8_ ? (hi4_ ? n2 : n0) : (hi4_ ? c2 : c0);                                \
        const uint32_t hi_ = hi8_ ? (hi4_ ? n3 : n1) : (hi4_ ? c3 : c1);                                \
        /* bytes 2s, 2s+1 of {hi, lo}: selector 0x0c0c0100 + 0x0202 * s */                              \
        const uint32_t code_ = __builtin_amdgcn_perm(hi_, lo_, 0x0c0c0100u + 0x0202u * ((at) & 3u));    \
        (dst) = order_entry(table, code_, (uint32_t)a.n_groups, (uint32_t)a.n_order);                   \
    } while (0)

// Decode step c of the ring at LDS byte address `wrow` (128 one-byte columns + 8 spare
// bytes): clear the half that becomes columns kend .. kend+63, then decode until every lane
// has passed column kend = 64 (c + 1); lanes that are there already keep going while their
// next codeword fits into the ring.  AFTER_WAIT runs right after the step's one wait for
// global memory (a good place to issue loads that should stay in flight for a whole step).
// A weight's ring byte is its two-bit field (2: +1, 6: -1) shifted left by BYTE_SHIFT.
#define QMOE_RING_DECODE_STEP(c, AFTER_WAIT, BYTE_SHIFT)                                                          \
    const int kc = (c) * kMmKc, kend = kc + kMmKc;                                                      \
    _Pragma("unroll") for (int i_ = 0; i_ < kMmKc / 8; i_++)                                            \
        ((lw_u64)(uintptr_t)(wrow + (uint32_t)((((c) + 1) & 1) * kMmKc)))[i_] = 0ull;                   \
    do {                                                                                                \
        /* Slide the window by one piece where its first half is used up (once per step as a */        \
        /* rule; the loop comes back only for lanes that use up a whole window in one step). */        \
        /* The other lanes fetch the piece they already wait for again, so that the load is */         \
        /* unconditional and stays in flight until the next slide. */                                   \
        {                                                                                               \
            const bool s8_ = sub >= 8u;                                                                 \
            sub -= s8_ ? 8u : 0u;                                                                       \
            pp += s8_ ? 16u : 0u;                                                                       \
            const uint32_t f0_ = fut.x, f1_ = fut.y, f2_ = fut.z, f3_ = fut.w;                          \
            c0 = s8_ ? n0 : c0; c1 = s8_ ? n1 : c1; c2 = s8_ ? n2 : c2; c3 = s8_ ? n3 : c3;             \
            n0 = s8_ ? f0_ : n0; n1 = s8_ ? f1_ : n1; n2 = s8_ ? f2_ : n2; n3 = s8_ ? f3_ : n3;         \
            fut = *(gp_u32x4)(pp + 32u < last ? pp + 32u : last);                                       \
        }                                                                                               \
        AFTER_WAIT                                                                                      \
        /* No branches inside the inner loop: a lane that sits out decodes an empty entry into */      \
        /* the spare bytes after its ring.  The look-up of the next codeword is issued before */       \
        /* the current one is applied. */                                                               \
        uint32_t ent_next_;                                                                             \
        QMOE_MM_ENTRY_AT(ent_next_, sub);                                                               \
        while (__any(left != 0u && pos < kend && sub < 16u)) {                                          \
            const bool go_ = left != 0u && pos <= kc + kMmAhead && sub < 16u;                           \
            const uint32_t ent_ = go_ ? ent_next_ : 0u;                                                 \
            left -= go_ ? 1u : 0u;                                                                      \
            sub += go_ ? 1u : 0u;                                                                       \
            QMOE_MM_ENTRY_AT(ent_next_, sub);                                                           \
            const uint32_t base_ = go_ ? (uint32_t)pos : (uint32_t)kMmRing;                             \
            const uint32_t mask_ = go_ ? (uint32_t)(kMmRing - 1) : 0xFFu;                               \
            /* fields are right-aligned in device-order entries: an unused one (0) comes first */      \
            /* and writes a zero at the run's first column, before any real weight */                   \
            _Pragma("unroll") for (int z_ = 0; z_ < kRunMaxNonzeros; z_++) {                            \
                const uint32_t f_ = (ent_ >> (8 + 8 * z_)) & 0xFFu;                                     \
                const uint32_t col_ = (base_ + (f_ >> 3)) & mask_;                                      \
                /* shift 5: 0, 0x40 (+2.0), 0xC0 (-2.0) */                                              \
                *(lw_u8)(uintptr_t)(wrow + col_) = (unsigned char)((f_ & 6u) << (BYTE_SHIFT));          \
            }                                                                                           \
            pos += (int)((ent_ & 0xFFu) >> 3);                                                          \
        }                                                                                               \
    } while (__any(left != 0u && pos < kend))

// MB: 32-token blocks in the tile (1 or 2).  wt / xt: LDS byte addresses of the weight
// rings and the two activation buffers.
template <int MB, int EPI, int ASYM>
__device__ __forceinline__ void mm_item(const ProductArgs &a, const qmoe_matrix &M, int blk, int slot0, int ntok,
                                        lp_u32 table, uint32_t wt, uint32_t xt, lp_i32 tok_ids, lp_f32 gate_s,
                                        int lag)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;

    // this thread's part of the activation tile: token tx, columns 8*seg .. 8*seg+7 of each step
    const int tx = tid >> 3, seg = tid & 7;
    const bool x_live = tx < ntok;
    size_t xrow = 0;
    if (x_live) {
        const int tok = a.perm ? a.perm[slot0 + tx] : slot0 + tx;
        xrow = a.x_by_slot ? (size_t)(slot0 + tx) : (size_t)tok;
    }
    // Loads are unconditional (a lane without a token, or past the last column, reads a
    // valid address and drops the value when it stages it): a load under a branch would
    // be waited for at the end of the branch instead of staying in flight.
    const bool x_ok = x_live && 8 * seg + 8 <= a.cols;
    const uintptr_t xsrc =
        reinterpret_cast<uintptr_t>(a.x) + (x_ok ? 2 * (xrow * (size_t)a.ldx + 8 * (size_t)seg) : (size_t)0);
    const int x_last = x_ok ? a.cols - 8 * seg - 8 : 0;  // last column offset this thread may read at
    auto load_x = [&](int kc) -> u32x4 { return *(gp_u32x4)(xsrc + 2 * (uintptr_t)min(kc, x_last)); };
    auto keep_x = [&](const u32x4 &v, int kc) -> u32x4 {
        return (x_ok && kc <= x_last) ? v : u32x4{0u, 0u, 0u, 0u};
    };
    const uint32_t x_slot = xt + (uint32_t)(tx * kMmXRowBytes + 16 * seg);  // in buffer 0

    // this lane's row and its codewords
    const int r0 = blk * a.mm_rows_per_block;
    const int row = r0 + tid;
    const bool row_live = tid < a.mm_rows_per_block && row < a.rows;
    QMOE_RING_ROW_SETUP(M, row, row_live);
    const uint32_t wrow = wt + (uint32_t)(tid * kMmWRowBytes);

    f32x16 acc[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; mb++)
#pragma unroll
        for (int nb = 0; nb < 2; nb++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[mb][nb][v] = 0.0f;

    // Activations: step c is read from LDS buffer c & 1; step c + 1 is in flight to a
    // register during step c and staged at its end.
    *(lw_u32x4)(uintptr_t)x_slot = keep_x(load_x(0), 0);
    u32x4 xr = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < kMmKc / 8; i++) ((lw_u64)(uintptr_t)wrow)[i] = 0ull;

    // asymmetric grid: the grid points of the two rows whose weights this lane feeds to the matrix cores
    uint32_t g_hi[2] = {0u, 0u}, g_lo[2] = {0u, 0u};
    if constexpr (ASYM) {
#pragma unroll
        for (int nb = 0; nb < 2; nb++) {
            const int rl = 64 * wave + 32 * nb + l32;
            uint32_t pair = 0u;  // a row past the end, or a matrix without a pair array, multiplies as zeros
            if (rl < a.mm_rows_per_block && r0 + rl < a.rows && M.minmax_bf16) pair = ((gp_u32)M.minmax_bf16)[r0 + rl];
            g_hi[nb] = pair << 16;
            g_lo[nb] = pair & 0xFFFF0000u;
        }
    }
    const uint32_t wfrag = wt + (uint32_t)((64 * wave + l32) * kMmWRowBytes + 8 * lhi);
    const uint32_t xfrag0 = xt + (uint32_t)(l32 * kMmXRowBytes + 16 * lhi);
    const int nsteps = (a.cols + kMmKc - 1) / kMmKc;

    // The two wavefronts that share a SIMD work half a step apart, so that one decodes
    // (vector ALU, LDS) while the other multiplies (matrix cores): both run the same
    // sequence -- decode, barrier, multiply and stage, barrier -- but the trailing one
    // (lag 1) passes one barrier before it starts and the leading one passes one after it
    // has finished.
    __syncthreads();  // token ids, gates and the first activation step are in place
    if (lag != 0) lds_barrier();
    for (int c = 0; c < nsteps; c++) {
        // ---- decode step c; the next step's activations, staged after this step's product,
        // are fetched right after the window's wait, so that a whole step hides the latency
        // of both loads (the empty asm keeps the compiler from moving the load up, in front
        // of that wait)
        // The arbiter serves the older wavefront of a SIMD first, so the older four finish a
        // step's decoding early and wait at the step's barrier (a quarter of their time) for
        // the younger four; the younger ones decode at a raised priority (2-3 %, measured;
        // raising it for all eight helps the second product only, alternating it hurts).
        if (wave >= kMmThreads / 128) __builtin_amdgcn_s_setprio(1);
        QMOE_RING_DECODE_STEP(c, {
            int k_next = kend;
            asm volatile("" : "+s"(k_next));
            xr = load_x(k_next);
        }, ASYM ? 0 : 5);
        __builtin_amdgcn_s_setprio(0);
        // the rows this wavefront multiplies are the ones its own lanes wrote
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (a.mm_stagger) lds_barrier();

        // ---- multiply step c
        const uint32_t xf = xfrag0 + (uint32_t)((c & 1) * kMmTokens * kMmXRowBytes);
        const uint32_t wf = wfrag + (uint32_t)((c & 1) * kMmKc);
#pragma unroll
        for (int ks = 0; ks < kMmKc / 16; ks++) {
            bf16x8 bw[2], ax[MB];
#pragma unroll
            for (int nb = 0; nb < 2; nb++) {
                const unsigned long long d = *(lp_u64)(uintptr_t)(wf + (uint32_t)(nb * 32 * kMmWRowBytes + 16 * ks));
                if constexpr (ASYM)
                    bw[nb] = mm_expand_minmax((uint32_t)d, (uint32_t)(d >> 32), g_hi[nb], g_lo[nb]);
                else
                    bw[nb] = mm_expand((uint32_t)d, (uint32_t)(d >> 32));
            }
#pragma unroll
            for (int mb = 0; mb < MB; mb++) {
                const u32x4 t = *(lp_u32x4)(uintptr_t)(xf + (uint32_t)(mb * 32 * kMmXRowBytes + 32 * ks));
                __builtin_memcpy(&ax[mb], &t, 16);
            }
#pragma unroll
            for (int mb = 0; mb < MB; mb++)
#pragma unroll
                for (int nb = 0; nb < 2; nb++)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax[mb], bw[nb], acc[mb][nb], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- stage this thread's part of step c + 1 of the activations: the buffer held
        // step c - 1, which every wavefront has finished by now (the trailing ones one
        // barrier ago), and nobody reads step c + 1 before two more barriers
        *(lw_u32x4)(uintptr_t)(x_slot + (uint32_t)(((c + 1) & 1) * kMmTokens * kMmXRowBytes)) =
            keep_x(xr, kend);
        lds_barrier();
    }
    if (lag == 0) lds_barrier();

    // accumulator v of lane l: token 32*mb + 8*(v/4) + 4*(l/32) + v%4, row 32*nb + l%32 of the wavefront's 64
#pragma unroll
    for (int nb = 0; nb < 2; nb++) {
        const int rl = 64 * wave + 32 * nb + l32;
        const int r = r0 + rl;
        if (rl < a.mm_rows_per_block && r < a.rows) {
            // symmetric grid: the weights were +-2; asymmetric: they were the grid points themselves
            const float scale = ASYM ? 1.0f : 0.5f * half_bits_to_float(((gp_u16)M.scale_f16)[r]);
#pragma unroll
            for (int mb = 0; mb < MB; mb++) {
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    const int t = 32 * mb + 8 * (v / 4) + 4 * lhi + (v % 4);
                    if (t < ntok) {
                        const float val = acc[mb][nb][v] * scale;
                        if constexpr (EPI == 0) {
                            reinterpret_cast<float *>(a.out)[(size_t)tok_ids[t] * a.ld_out + r] = gate_s[t] * val;
                        } else {
                            const float h = val > 0.0f ? val : 0.0f;
                            reinterpret_cast<uint16_t *>(a.out)[(size_t)(slot0 + t) * a.ld_out + r] =
                                float_to_bf16_bits(h);
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
    unsigned char *wt = smem + table_bytes;                           // [512][kMmWRowBytes]
    unsigned char *xt = wt + (size_t)kMmThreads * kMmWRowBytes;       // 2 x [64][kMmXRowBytes]
    int *tok_ids = reinterpret_cast<int *>(xt + 2 * (size_t)kMmTokens * kMmXRowBytes);  // [64]
    float *gate_s = reinterpret_cast<float *>(tok_ids + kMmTokens);   // [64]
    int *next_item = reinterpret_cast<int *>(gate_s + kMmTokens);     // [1]

    // A layer call brings a list of (expert, token tile) items and a device counter that hands
    // them out; the single-matrix call has neither: its items are the tiles of 64 consecutive
    // tokens of `single`, dealt out round robin.
    const bool listed = a.items != nullptr;
    const int n_items = listed ? min(*a.n_items_dev, a.max_items) : (a.batch + kMmTokens - 1) / kMmTokens;
    const int total = (int)min((long long)n_items * a.mm_row_blocks, 0x7FFFFFFFLL);
    if (total <= 0 || (!listed && (int)blockIdx.x >= total)) return;
    stage_words(table_w, a.order_table, a.n_order);

    // Order of arrival of this wavefront on its SIMD (SIMD_ID: bits 5:4 of HW_ID): the
    // first and the second wavefront of a SIMD take opposite halves of the step.  (The
    // tile's first bytes serve as counters; the first item clears them again.)
    int lag = 0;
    if (a.mm_stagger) {
        int *simd_count = reinterpret_cast<int *>(wt);
        if (threadIdx.x < 4) simd_count[threadIdx.x] = 0;
        __syncthreads();
        const int simd = (int)__builtin_amdgcn_s_getreg(4 | (4 << 6) | (1 << 11));
        int rank = 0;
        if ((threadIdx.x & 63) == 0) rank = atomicAdd(&simd_count[simd & 3], 1);
        lag = __builtin_amdgcn_readfirstlane(rank) & 1;
    }

    int g_static = (int)blockIdx.x;
    for (;;) {
        __syncthreads();  // everyone is done with the previous item
        if (threadIdx.x == 0) {
            const int g = listed ? atomicAdd(a.work_counter, 1) : g_static;
            *next_item = g < total ? g : -1;
        }
        g_static += (int)gridDim.x;
        __syncthreads();
        const int g = *next_item;
        if (g < 0) break;
        const int idx = g / a.mm_row_blocks;
        const int blk = g - idx * a.mm_row_blocks;
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
        if (threadIdx.x < kMmTokens) {
            const int t = threadIdx.x;
            const int tok = t < ntok ? (a.perm ? a.perm[slot0 + t] : slot0 + t) : 0;
            tok_ids[t] = tok;
            gate_s[t] = (a.gate && t < ntok) ? a.gate[tok] : 1.0f;
        }
        const qmoe_matrix M = a.mats ? a.mats[expert] : a.single;
        const uint32_t wt_addr = (uint32_t)(uintptr_t)(lw_u8)wt, xt_addr = (uint32_t)(uintptr_t)(lw_u8)xt;
        if (ntok <= 32)
            mm_item<1, EPI, ASYM>(a, M, blk, slot0, ntok, (lp_u32)table_w, wt_addr, xt_addr, (lp_i32)tok_ids,
                            (lp_f32)gate_s, lag);
        else
            mm_item<2, EPI, ASYM>(a, M, blk, slot0, ntok, (lp_u32)table_w, wt_addr, xt_addr, (lp_i32)tok_ids,
                            (lp_f32)gate_s, lag);
    }
}

// ---------------------------------------------------------------- one matrix, a few tokens: a row per 16 lanes
//
// A single matrix gives the lane-per-row kernel above a few thousand lanes, each walking a
// whole row codeword by codeword: fine for throughput over hundreds of experts, slow as the
// latency of one product.  Here 16 lanes (a DPP row) share a matrix row: every lane takes
// one codeword of the next 16, the running column index of the sequential decoder becomes
// an inclusive prefix sum of the 16 run lengths (four DPP row shifts, the previous step's
// total carried in through lane 0), each lane gathers the activations of its own run, and
// the 16 partial sums are added in a fixed order at the row's end.  rows x 16 lanes keep the
// whole GPU busy with one matrix.  The table is read from L2 (no 65 KB staging per
// workgroup: the launch is over in microseconds).
template <bool RUN, int ASYM>
__global__ __launch_bounds__(256) void k_matvec_rows(const ProductArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *xs_w = reinterpret_cast<uint16_t *>(smem);
    const uint32_t xs_addr = (uint32_t)(uintptr_t)(lp_u16)xs_w;
    constexpr int DICT = RUN ? kDictRun : kDictWords;
    const qmoe_matrix M = a.single;
    const int l16 = threadIdx.x & 15, grp = threadIdx.x >> 4, ngrp = blockDim.x >> 4;
    const int row_blocks = (a.rows + ngrp - 1) / ngrp;
    const int n_tiles = (a.batch + a.tb_max - 1) / a.tb_max;
    const long long total = (long long)n_tiles * row_blocks;
    int cur_tile = -1, ntok = 0, slot0 = 0, tbi = 1;
    for (long long g = blockIdx.x; g < total; g += gridDim.x) {
        const int tile = (int)(g / row_blocks);
        const int rb = (int)(g - (long long)tile * row_blocks);
        if (tile != cur_tile) {
            __syncthreads();  // everyone is done with the previous tile's activations
            slot0 = tile * a.tb_max;
            ntok = min(a.tb_max, a.batch - slot0);
            tbi = ntok <= 1 ? 1 : (ntok <= 2 ? 2 : (ntok <= 4 ? 4 : 8));
            auto row_of = [&](int t) { return slot0 + t; };
            switch (tbi) {
            case 1: stage_x_one(xs_w, a.x + (size_t)slot0 * a.ldx, a.cols, true, false); break;  // lds_load_x<1> reads the +x slot
            case 2: stage_x_tile<2>(xs_w, a.x, row_of, ntok, a.ldx, a.cols); break;
            case 4: stage_x_tile<4>(xs_w, a.x, row_of, ntok, a.ldx, a.cols); break;
            default: stage_x_tile<8>(xs_w, a.x, row_of, ntok, a.ldx, a.cols); break;
            }
            __syncthreads();
            cur_tile = tile;
        }
        const int r = rb * ngrp + grp;
        if (r >= a.rows) continue;
        const uint32_t kend = min(min(M.row_off[r + 1], M.n_codes), kMaxCodes);
        const uint32_t kbeg = min(M.row_off[r], kend);
        // y = scale * (signed sum) + mid * (sum under |weight|); mid = 0 on the symmetric grid
        float scale, mid = 0.0f;
        if constexpr (ASYM) {
            const uint32_t pair = reinterpret_cast<const uint32_t *>(M.minmax_bf16)[r];
            const float w_min = __uint_as_float(pair << 16), w_max = __uint_as_float(pair & 0xFFFF0000u);
            scale = 0.5f * (w_max - w_min);
            mid = 0.5f * (w_max + w_min);
        } else {
            scale = half_bits_to_float(M.scale_f16[r]);
        }
        auto row = [&](auto tag) {
            constexpr int TBI = decltype(tag)::value;
            constexpr int NA = TBI * (1 + ASYM);
            float acc[NA];
#pragma unroll
            for (int t = 0; t < NA; t++) acc[t] = 0.0f;
            int incl = 0;
            for (uint32_t kb = kbeg; kb < kend; kb += 16) {
                const Step s = decode_step<RUN>(a, M.codes, kb + l16, kend, l16, incl);
                const Entry e{s.e0, s.e1};
                accumulate<TBI, DICT, ASYM>(e, xs_addr, 8u * (uint32_t)s.start, acc);
            }
#pragma unroll
            for (int t = 0; t < NA; t++) acc[t] = row_sum16_to_last(acc[t]);
            if (l16 == 15) {
#pragma unroll
                for (int t = 0; t < TBI; t++)
                    if (t < ntok) {
                        float v = acc[t] * scale;
                        if constexpr (ASYM) v = fmaf(acc[NA - TBI + t], mid, v);
                        reinterpret_cast<float *>(a.out)[(size_t)(slot0 + t) * a.ld_out + r] = v;
                    }
            }
        };
        switch (tbi) {
        case 1: row(std::integral_constant<int, 1>{}); break;
        case 2: row(std::integral_constant<int, 2>{}); break;
        case 4: row(std::integral_constant<int, 4>{}); break;
        default: row(std::integral_constant<int, 8>{}); break;
        }
    }
}

// ---------------------------------------------------------------- decompression of whole matrices
//
// The codec without the product: dense ternary (int8) or scaled bf16 copies of compressed
// matrices, for consumers that want a plain matrix (a library GEMM, a check).  Same ring
// decoder as the matrix-core product: a workgroup of 512 lanes owns up to 512 rows, one lane
// per row; after each 64-column step a wavefront writes out the 64 x 64 tile its own lanes
// decoded, 8 rows per store instruction with 8 lanes covering a row's 64 columns, so that
// the stores are whole 64- or 128-byte runs.  Wavefronts never wait for each other.

struct DecompressArgs {
    const qmoe_matrix *mats;  // device array
    void *const *out;         // device array of destinations (row-major rows x cols), nullptr = skip
    int n_mats, rows, cols;
    int rows_per_block, row_blocks;
    const uint32_t *order_table;
    int n_groups, n_order;
};

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
    const uint32_t wt = (uint32_t)(uintptr_t)(lw_u8)(smem + table_bytes);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wrow = wt + (uint32_t)(tid * kMmWRowBytes);
    const int seg = lane & 7, sub_row = lane >> 3;  // write-out role: columns 8*seg.., rows sub_row + 8*i
    const int nsteps = (a.cols + kMmKc - 1) / kMmKc;
    const long long total = (long long)a.n_mats * a.row_blocks;

    for (long long g = blockIdx.x; g < total; g += gridDim.x) {
        const int m = (int)(g / a.row_blocks);
        const int blk = (int)(g - (long long)m * a.row_blocks);
        unsigned char *out = static_cast<unsigned char *>(a.out[m]);
        if (!out) continue;
        const qmoe_matrix M = a.mats[m];
        const int r0 = blk * a.rows_per_block;
        const int row = r0 + tid;
        const bool row_live = tid < a.rows_per_block && row < a.rows;
        QMOE_RING_ROW_SETUP(M, row, row_live);
#pragma unroll
        for (int i = 0; i < kMmKc / 8; i++) ((lw_u64)(uintptr_t)wrow)[i] = 0ull;

        // bf16 scale of the eight rows this lane writes out, in both halves of a register
        uint32_t s2[8];
        if constexpr (OUT == 2) {
            // the (w_min, w_max) pair as stored: w_min in the low half
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const int rl = 64 * wave + sub_row + 8 * i;
                s2[i] = 0u;
                if (rl < a.rows_per_block && r0 + rl < a.rows && M.minmax_bf16) s2[i] = ((gp_u32)M.minmax_bf16)[r0 + rl];
            }
        }
        if constexpr (OUT == 1) {
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const int rl = 64 * wave + sub_row + 8 * i;
                uint32_t b = 0;
                if (rl < a.rows_per_block && r0 + rl < a.rows)
                    b = float_to_bf16_bits(half_bits_to_float(((gp_u16)M.scale_f16)[r0 + rl]));
                s2[i] = b | (b << 16);
            }
        }

        for (int c = 0; c < nsteps; c++) {
            QMOE_RING_DECODE_STEP(c, {}, OUT == 2 ? 0 : 5);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const int k = kc + 8 * seg;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const int rl = 64 * wave + sub_row + 8 * i;
                const int r = r0 + rl;
                if (rl < a.rows_per_block && r < a.rows && k + 8 <= a.cols) {
                    const unsigned long long d =
                        *(lp_u64)(uintptr_t)(wt + (uint32_t)(rl * kMmWRowBytes + (c & 1) * kMmKc + 8 * seg));
                    const uint32_t w0 = (uint32_t)d, w1 = (uint32_t)(d >> 32);
                    const size_t at = (size_t)r * a.cols + k;
                    if constexpr (OUT == 0) {
                        // ring byte 0x40 -> 0x01, 0xC0 -> 0xFF, 0 -> 0
                        const uint32_t o0 = ((w0 >> 6) & 0x01010101u) | (((w0 >> 7) & 0x01010101u) * 0xFEu);
                        const uint32_t o1 = ((w1 >> 6) & 0x01010101u) | (((w1 >> 7) & 0x01010101u) * 0xFEu);
                        *reinterpret_cast<unsigned long long *>(out + at) = (unsigned long long)o0 | ((unsigned long long)o1 << 32);
                    } else if constexpr (OUT == 2) {
                        const bf16x8 v = mm_expand_minmax(w0, w1, s2[i] << 16, s2[i] & 0xFFFF0000u);
                        u32x4 o;
                        __builtin_memcpy(&o, &v, 16);
                        *reinterpret_cast<u32x4 *>(out + 2 * at) = o;
                    } else {
                        u32x4 o;
#pragma unroll
                        for (int h = 0; h < 4; h++) {
                            // two ring bytes -> the high bytes of two 16-bit halves: 0x4000 / 0xC000 / 0
                            const uint32_t e = __builtin_amdgcn_perm(0u, h < 2 ? w0 : w1, (h & 1) ? 0x030c020cu : 0x010c000cu);
                            const uint32_t present = ((e >> 14) & 0x00010001u) * 0xFFFFu;
                            o[h] = ((e & 0x80008000u) | s2[i]) & present;
                        }
                        *reinterpret_cast<u32x4 *>(out + 2 * at) = o;
                    }
                }
            }
            // the next step clears this half of the ring: after these reads
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// ---------------------------------------------------------------- pure decompression

template <bool RUN>
__global__ __launch_bounds__(256) void k_decode_dense(const ProductArgs a, int8_t *out)
{
    const qmoe_matrix M = a.single;
    const int l16 = threadIdx.x & 15, grp = threadIdx.x >> 4, ngrp = blockDim.x >> 4;
    for (int r = blockIdx.x * ngrp + grp; r < a.rows; r += gridDim.x * ngrp) {
        const uint32_t kend = min(min(M.row_off[r + 1], M.n_codes), kMaxCodes);
        const uint32_t kbeg = min(M.row_off[r], kend);
        int8_t *orow = out + (size_t)r * a.cols;
        int incl = 0;
        for (uint32_t kb = kbeg; kb < kend; kb += 16) {
            const Step s = decode_step<RUN>(a, M.codes, kb + l16, kend, l16, incl);
            for (int j = 0; j < s.len; j++) {
                int v = 0;
                if constexpr (RUN) {
#pragma unroll
                    for (int z = 0; z < kRunMaxNonzeros; z++) {
                        const int sh = 8 + 8 * z;
                        const int pos = (int)((s.e0 >> (sh + 3)) & 31u);
                        const int wi = ((int)(s.e0 << (32 - (sh + 3)))) >> 30;
                        if (pos == j) v += wi;
                    }
                } else {
                    const uint32_t w = j < 14 ? s.e0 : s.e1;
                    const int sym = (int)((w >> (4 + 2 * (j % 14))) & 3u);
                    v = sym == 2 ? 1 : (sym == 1 ? -1 : 0);
                }
                if (s.start + j < a.cols) orow[s.start + j] = (int8_t)v;
            }
        }
    }
}

// ---------------------------------------------------------------- dispatch

struct DispatchArgs {
    const int *expert_idx;
    int n_tokens, n_experts;
    int *tok_off;   // [E+1]
    int *perm;      // [T]
    int *counters;  // [8]
    Item *items_wi, *items_wo, *items_mm;
    int tb_wi, tb_wo;
    int mm_min;     // experts with at least this many tokens go to the matrix-core kernel (tiles of 64)
    float *y;       // rows of dropped tokens are zeroed (may be nullptr)
    int d_model;
};

// exclusive prefix sum of one int per thread over the workgroup; `tmp` holds >= 32 ints
__device__ __forceinline__ int block_exclusive_scan(int v, int *tmp, int &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = (blockDim.x + 63) >> 6;
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) tmp[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        int w = lane < nwaves ? tmp[lane] : 0;
        int wi = w;
#pragma unroll
        for (int d = 1; d < 16; d <<= 1) {
            const int up = __shfl_up(wi, d, 64);
            if (lane >= d) wi += up;
        }
        if (lane < nwaves) tmp[lane] = wi - w;  // exclusive per wave
        if (lane == nwaves - 1) tmp[16] = wi;   // grand total
    }
    __syncthreads();
    const int base = tmp[wave];
    total = tmp[16];
    __syncthreads();
    return base + incl - v;
}

// The same for N values per thread at once (three barriers for all of them).
// `tmp` holds >= 17 * N ints.
template <int N>
__device__ __forceinline__ void block_exclusive_scan_n(const int (&v)[N], int *tmp, int (&excl)[N], int (&total)[N])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = (blockDim.x + 63) >> 6;
    int incl[N];
#pragma unroll
    for (int k = 0; k < N; k++) {
        incl[k] = v[k];
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl[k], d, 64);
            if (lane >= d) incl[k] += up;
        }
        if (lane == 63) tmp[wave * N + k] = incl[k];
    }
    __syncthreads();
    if (wave == 0) {
        // lane l: value l % N of wavefront l / N, for up to 64 / N wavefronts a turn
        for (int w0 = 0; w0 < nwaves; w0 += 64 / N) {
            const int k = lane % N, w = w0 + lane / N;
            const bool live = lane < (64 / N) * N && w < nwaves;
            const int mine = live ? tmp[w * N + k] : 0;
            int run = mine;  // inclusive over the wavefronts of this turn, same k: stride N lanes
#pragma unroll
            for (int d = N; d < 64; d <<= 1) {
                const int up = __shfl_up(run, d, 64);
                if (lane >= d) run += up;
            }
            const int carry = w0 ? tmp[16 * N + k] : 0;  // total of the turns before
            if (live) tmp[w * N + k] = carry + run - mine;
            __builtin_amdgcn_wave_barrier();
            // the last live wavefront of the turn leaves the running total
            const int last_w = min(nwaves, w0 + 64 / N) - 1;
            if (live && w == last_w) tmp[16 * N + k] = carry + run;
            __builtin_amdgcn_wave_barrier();
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < N; k++) {
        excl[k] = tmp[wave * N + k] + incl[k] - v[k];
        total[k] = tmp[16 * N + k];
    }
    __syncthreads();
}

// One workgroup of 1024 threads groups the tokens by expert (stable) and writes
// the work lists of both products.
__global__ __launch_bounds__(1024) void k_dispatch(const DispatchArgs a)
{
    extern __shared__ int sm[];
    int *cnt = sm;                 // [E] token count, later the write cursor of each expert
    int *tmp = sm + a.n_experts;   // [256] scan scratch, then two arrays of one round of tokens
    const int E = a.n_experts, T = a.n_tokens;
    const int tid = threadIdx.x, nthr = blockDim.x;

    // Tokens without an expert get a zero output row.  They are collected in a list (the two
    // arrays the scatter uses later) and their rows are cleared by whole wavefronts; a thread
    // clears a row alone only when the list is full.
    int *bad_list = tmp + 256, *n_bad = tmp + 255;
    const int bad_cap = 2 * nthr;
    for (int e = tid; e < E; e += nthr) cnt[e] = 0;
    if (tid == 0) *n_bad = 0;
    __syncthreads();
    int dropped = 0;
    for (int t = tid; t < T; t += nthr) {
        const int e = a.expert_idx[t];
        if (e >= 0 && e < E) {
            atomicAdd(&cnt[e], 1);
        } else {
            dropped++;
            if (a.y) {
                const int slot = atomicAdd(n_bad, 1);
                if (slot < bad_cap) {
                    bad_list[slot] = t;
                } else {
                    for (int c = 0; c < a.d_model; c++) a.y[(size_t)t * a.d_model + c] = 0.0f;
                }
            }
        }
    }
    __syncthreads();
    if (a.y) {
        const int nb = min(*n_bad, bad_cap);
        for (int i = tid >> 6; i < nb; i += nthr >> 6) {
            float *row = a.y + (size_t)bad_list[i] * a.d_model;
            for (int c = tid & 63; c < a.d_model; c += 64) row[c] = 0.0f;
        }
        __syncthreads();  // the list's memory is used again below
    }

    // each thread owns a contiguous chunk of experts
    const int chunk = (E + nthr - 1) / nthr;
    const int e0 = min(E, tid * chunk), e1 = min(E, e0 + chunk);
    // Work items of the scalar products are listed longest first (tiles of more than four
    // tokens, then of three or four, of two, of one): handed out in that order, the last
    // workgroups to finish are busy with short items.
    auto tile_class = [](int n) { return n > 4 ? 0 : (n > 2 ? 1 : (n == 2 ? 2 : 3)); };
    int s_tok = 0, s_act = 0, s_mm = 0;
    int s_wi[4] = {0, 0, 0, 0}, s_wo[4] = {0, 0, 0, 0};
    for (int e = e0; e < e1; e++) {
        const int n = cnt[e];
        s_tok += n;
        s_act += n > 0;
        if (n >= a.mm_min) {
            s_mm += (n + kMmTokens - 1) / kMmTokens;
        } else if (n > 0) {
            s_wi[tile_class(a.tb_wi)] += n / a.tb_wi;
            if (n % a.tb_wi) s_wi[tile_class(n % a.tb_wi)]++;
            s_wo[tile_class(a.tb_wo)] += n / a.tb_wo;
            if (n % a.tb_wo) s_wo[tile_class(n % a.tb_wo)]++;
        }
    }
    // all twelve sums in one scan
    const int sums[12] = {s_tok, s_act, s_mm, dropped, s_wi[0], s_wi[1], s_wi[2], s_wi[3],
                          s_wo[0], s_wo[1], s_wo[2], s_wo[3]};
    int before[12], all[12];
    block_exclusive_scan_n<12>(sums, tmp, before, all);
    int p_tok = before[0], p_mm = before[2];
    const int tot_tok = all[0], tot_act = all[1], tot_mm = all[2], tot_drop = all[3];
    int p_wi[4], p_wo[4], tot_wi = 0, tot_wo = 0;
#pragma unroll
    for (int k = 0; k < 4; k++) {
        p_wi[k] = tot_wi + before[4 + k];
        p_wo[k] = tot_wo + before[8 + k];
        tot_wi += all[4 + k];
        tot_wo += all[8 + k];
    }
    for (int e = e0; e < e1; e++) {
        const int n = cnt[e];
        a.tok_off[e] = p_tok;
        if (n >= a.mm_min) {
            for (int i = 0; i * kMmTokens < n; i++)
                a.items_mm[p_mm++] = Item{e, p_tok + i * kMmTokens, min(kMmTokens, n - i * kMmTokens), 0};
        } else {
            for (int i = 0; i * a.tb_wi < n; i++) {
                const int m = min(a.tb_wi, n - i * a.tb_wi);
                a.items_wi[p_wi[tile_class(m)]++] = Item{e, p_tok + i * a.tb_wi, m, 0};
            }
            for (int i = 0; i * a.tb_wo < n; i++) {
                const int m = min(a.tb_wo, n - i * a.tb_wo);
                a.items_wo[p_wo[tile_class(m)]++] = Item{e, p_tok + i * a.tb_wo, m, 0};
            }
        }
        cnt[e] = p_tok;  // becomes the expert's write cursor
        p_tok += n;
    }
    if (tid == 0) {
        a.tok_off[E] = tot_tok;
        a.counters[0] = tot_tok;
        a.counters[1] = tot_drop;
        a.counters[2] = tot_act;
        a.counters[3] = tot_wi;
        a.counters[4] = tot_wo;
        a.counters[5] = 0; a.counters[6] = 0;  // work hand-out of the two scalar products
        a.counters[7] = tot_mm;
        a.counters[8] = 0; a.counters[9] = 0;  // work hand-out of the two matrix-core products
        for (int i = 10; i < kLayerCounters; i++) a.counters[i] = 0;
    }
    __syncthreads();

    // Stable scatter.  A wavefront takes 64 consecutive tokens; inside it a token's
    // rank among equal experts is counted by broadcasting every lane once.  The chunks of
    // 64 tokens must then take their places one after the other, in token order: one
    // wavefront walks the chunks of a round (no workgroup barrier between them), reads each
    // token's expert cursor and moves the cursors on; after that every thread stores its
    // own token.
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthr >> 6;
    int *tok_e = tmp + 256;          // [nthr] expert of the round's tokens (-1: none)
    int *tok_rs = tok_e + nthr;      // [nthr] rank | same << 8, later the token's slot
    for (int base = 0; base < T; base += nthr) {
        const int t = base + tid;
        int e = -1;
        if (t < T) {
            e = a.expert_idx[t];
            if (e < 0 || e >= E) e = -1;
        }
        int rank = 0, same = 0;
#pragma unroll 8
        for (int j = 0; j < 64; j++) {
            const int ej = __builtin_amdgcn_readlane(e, j);  // j is uniform: a scalar read, no LDS crossbar
            const int m = (ej == e) ? 1 : 0;
            same += m;
            rank += (j < lane) ? m : 0;
        }
        tok_e[tid] = e;
        tok_rs[tid] = rank | (same << 8);
        __syncthreads();
        if (wave == 0) {
            for (int w = 0; w < nwaves; w++) {
                const int ew = tok_e[64 * w + lane], rs = tok_rs[64 * w + lane];
                const int rk = rs & 0xFF, sm_ = rs >> 8;
                int cur = 0;
                if (ew >= 0) cur = cnt[ew];
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();  // every lane has read its cursor
                if (ew >= 0) {
                    tok_rs[64 * w + lane] = cur + rk;
                    if (rk == sm_ - 1) cnt[ew] = cur + sm_;
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();  // the cursors are moved before the next chunk reads them
            }
        }
        __syncthreads();
        if (e >= 0) a.perm[tok_rs[tid]] = t;
        __syncthreads();  // the round's arrays are free again
    }
}

// ---------------------------------------------------------------- encoder
//
// Longest-prefix coding of ternary rows with the dictionary's trie (Section 4.3.3
// "Encoding"), one row per lane: walk pairs from the root while a child exists, emit the
// codeword of the deepest node that ends an entry, continue after that entry.  Three
// launches: count codewords per row, turn the counts into row offsets (one workgroup), write
// the codewords.  Same stream as qmoe_encode_host, codeword for codeword.

struct EncodeArgs {
    const int8_t *tern;   // [rows][cols], values -1 / 0 / +1
    int rows, cols;
    const int32_t *child, *code;
    uint32_t *row_off;    // [rows+1]
    uint16_t *codes;
    unsigned long long codes_cap;
    int *status;          // [2]: first error (qmoe_status, 0 = none), a row it happened in
};

template <bool WRITE>
__global__ __launch_bounds__(256) void k_encode(const EncodeArgs a)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= a.rows) return;
    if (WRITE && a.status[0] != 0) return;
    const int8_t *row = a.tern + (size_t)r * a.cols;
    const int np = a.cols / 2;
    const size_t out = WRITE ? (size_t)a.row_off[r] : 0;
    uint32_t n = 0;
    int bad = 0;
    int i = 0;
    while (i < np) {
        int node = 0, best = -1, best_len = 0, depth = 0;
        while (i + depth < np) {
            const int va = row[2 * (i + depth)], vb = row[2 * (i + depth) + 1];
            if (va < -1 || va > 1 || vb < -1 || vb > 1) { bad = QMOE_E_BAD_SYMBOL; break; }
            // value -> symbol: 0 -> 0, -1 -> 1, +1 -> 2; pair index = 3 * first + second
            const int sa = va == 0 ? 0 : (va < 0 ? 1 : 2), sb = vb == 0 ? 0 : (vb < 0 ? 1 : 2);
            const int nx = a.child[(size_t)node * 9 + 3 * sa + sb];
            if (nx < 0) break;
            node = nx;
            depth++;
            const int c = a.code[node];
            if (c >= 0) { best = c; best_len = depth; }
        }
        if (bad) break;
        if (best < 0) { bad = QMOE_E_UNENCODABLE; break; }
        if (WRITE) a.codes[out + n] = (uint16_t)best;
        n++;
        i += best_len;
    }
    if (bad) {
        if (atomicCAS(&a.status[0], 0, bad) == 0) a.status[1] = r;
        n = 0;
    }
    if (!WRITE) a.row_off[r + 1] = n;
}

// counts in row_off[1..rows] -> offsets; one workgroup
__global__ __launch_bounds__(1024) void k_encode_offsets(const EncodeArgs a)
{
    __shared__ int tmp[32];
    unsigned long long base = 0;
    if (threadIdx.x == 0) a.row_off[0] = 0;
    for (int r0 = 0; r0 < a.rows; r0 += (int)blockDim.x) {
        const int r = r0 + (int)threadIdx.x;
        const int c = r < a.rows ? (int)a.row_off[r + 1] : 0;
        int total;
        const int excl = block_exclusive_scan(c, tmp, total);
        if (r < a.rows) a.row_off[r + 1] = (uint32_t)(base + (unsigned long long)(excl + c));
        base += (unsigned long long)total;
    }
    if (threadIdx.x == 0 && (base > a.codes_cap || base > 0xFFFFFFFFull)) atomicCAS(&a.status[0], 0, QMOE_E_BUFFER_TOO_SMALL);
}

// ---------------------------------------------------------------- uncompressed bf16 comparator

struct DenseArgs {
    const uint16_t *const *mats;  // device array of row-major bf16 matrices, by expert
    const Item *items;
    const int *n_items_dev;
    int max_items, n_experts;
    const int *perm;
    const uint16_t *x;
    int x_by_slot, ldx;
    void *out;
    int ld_out;
    const float *gate;
    int epilogue;
    int rows, cols, rows_per_item, blocks_per_pass, tb_max;
    int *work_counter;  // zeroed by the dispatch kernel
};

// One wavefront per row; a lane takes four consecutive columns at a time (8 bytes of
// weights, coalesced to 512 bytes per wavefront) and the matching activations from
// token-major fp32 planes in LDS (16 bytes per lane, consecutive lanes: conflict-free).
template <int TBI>
__device__ __forceinline__ void dense_rows(const DenseArgs &a, const uint16_t *W, int ntok, int slot0,
                                           int r0, int r1, const float *xs, int plane, const int *tok_ids)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int nq = a.cols / 4;
    for (int r = r0 + wave; r < r1; r += nwaves) {
        const uint2 *wrow = reinterpret_cast<const uint2 *>(W + (size_t)r * a.cols);
        float acc[TBI];
#pragma unroll
        for (int t = 0; t < TBI; t++) acc[t] = 0.0f;
#pragma unroll 4
        for (int c4 = lane; c4 < nq; c4 += 64) {
            const uint2 q = wrow[c4];
            const float w0 = __uint_as_float(q.x << 16), w1 = __uint_as_float(q.x & 0xFFFF0000u);
            const float w2 = __uint_as_float(q.y << 16), w3 = __uint_as_float(q.y & 0xFFFF0000u);
#pragma unroll
            for (int t = 0; t < TBI; t++) {
                const float4 x = reinterpret_cast<const float4 *>(xs + (size_t)t * plane)[c4];
                acc[t] = fmaf(w3, x.w, fmaf(w2, x.z, fmaf(w1, x.y, fmaf(w0, x.x, acc[t]))));
            }
        }
#pragma unroll
        for (int t = 0; t < TBI; t++) {
#pragma unroll
            for (int d = 32; d > 0; d >>= 1) acc[t] += __shfl_down(acc[t], d, 64);
        }
        if (lane == 0) {
#pragma unroll
            for (int t = 0; t < TBI; t++) {
                if (t < ntok) {
                    if (a.epilogue == 0) {
                        const int tok = tok_ids[t];
                        const float g = a.gate ? a.gate[tok] : 1.0f;
                        reinterpret_cast<float *>(a.out)[(size_t)tok * a.ld_out + r] = g * acc[t];
                    } else {
                        const float h = acc[t] > 0.0f ? acc[t] : 0.0f;
                        reinterpret_cast<uint16_t *>(a.out)[(size_t)(slot0 + t) * a.ld_out + r] =
                            float_to_bf16_bits(h);
                    }
                }
            }
        }
    }
}

__global__ __launch_bounds__(1024) void k_dense_bf16(const DenseArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float *xs = reinterpret_cast<float *>(smem);
    const int plane = (a.cols + 3) / 4 * 4;  // one token's activations
    const size_t xs_bytes = (size_t)plane * a.tb_max * sizeof(float);
    int *tok_ids = reinterpret_cast<int *>(smem + xs_bytes);
    int *x_rows = tok_ids + kMaxTokenTile;
    int *next_item = x_rows + kMaxTokenTile;

    const int n_pass = min(*a.n_items_dev, a.max_items);
    const int total = (int)min((long long)n_pass * a.blocks_per_pass, 0x7FFFFFFFLL);
    int cur_pass = -1, ntok = 0, slot0 = 0, expert = 0, tbi = 1;
    for (;;) {
        __syncthreads();
        if (threadIdx.x == 0) {
            const int g = atomicAdd(a.work_counter, 1);
            *next_item = g < total ? g : -1;
        }
        __syncthreads();
        const int g = *next_item;
        if (g < 0) break;
        const int pass = g / a.blocks_per_pass;
        const int blk = g - pass * a.blocks_per_pass;
        if (pass != cur_pass) {
            const Item it = a.items[pass];
            expert = it.expert; slot0 = it.slot0; ntok = it.ntok;
            if (expert < 0 || expert >= a.n_experts || ntok < 1) ntok = 0;
            ntok = min(ntok, a.tb_max);
            tbi = ntok <= 1 ? 1 : (ntok <= 2 ? 2 : (ntok <= 4 ? 4 : 8));
            if (threadIdx.x < kMaxTokenTile) {
                const int t = threadIdx.x;
                int tok = 0, xr = 0;
                if (t < ntok) {
                    tok = a.perm[slot0 + t];
                    xr = a.x_by_slot ? slot0 + t : tok;
                }
                tok_ids[t] = tok;
                x_rows[t] = xr;
            }
            __syncthreads();
            for (int t = 0; t < tbi; t++)
                for (int c = threadIdx.x; c < plane; c += blockDim.x) {
                    float v = 0.0f;
                    if (c < a.cols && t < ntok) v = bf16_bits_to_float(a.x[(size_t)x_rows[t] * a.ldx + c]);
                    xs[(size_t)t * plane + c] = v;
                }
            __syncthreads();
            cur_pass = pass;
        }
        if (ntok == 0) continue;
        const uint16_t *W = a.mats[expert];
        if (W == nullptr) continue;
        const int r0 = blk * a.rows_per_item;
        const int r1 = min(a.rows, r0 + a.rows_per_item);
        switch (tbi) {
        case 1: dense_rows<1>(a, W, ntok, slot0, r0, r1, xs, plane, tok_ids); break;
        case 2: dense_rows<2>(a, W, ntok, slot0, r0, r1, xs, plane, tok_ids); break;
        case 4: dense_rows<4>(a, W, ntok, slot0, r0, r1, xs, plane, tok_ids); break;
        default: dense_rows<8>(a, W, ntok, slot0, r0, r1, xs, plane, tok_ids); break;
        }
    }
}

// ---------------------------------------------------------------- plain streaming copy

// 16 bytes per lane per iteration, grid-stride; the yardstick for what a kernel
// that only moves bytes reaches on this GPU, and the calibration of the HBM counters.
__global__ __launch_bounds__(256) void k_stream_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------- stream renumbering

// codes[i] = map[codes[i]], in place (interchange numbering -> device numbering)
__global__ __launch_bounds__(256) void k_renumber(uint16_t *codes, size_t n, const uint16_t *__restrict__ map)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) codes[i] = map[codes[i]];
}

// ---------------------------------------------------------------- launch helpers

struct DeviceInfo {
    int cus = 0;
    int max_lds = 0;
    bool ok = false;
};

qmoe_status device_info(DeviceInfo *out)
{
    static DeviceInfo cached[64];
    int dev = 0;
    QMOE_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return QMOE_E_LIMIT;
    if (!cached[dev].ok) {
        int cus = 0, lds = 0;
        QMOE_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        QMOE_HIP_TRY(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
        cached[dev].cus = cus;
        cached[dev].max_lds = lds;
        cached[dev].ok = true;
    }
    *out = cached[dev];
    return QMOE_OK;
}

// A side stream and two events per device, made on first use and kept until the process
// ends: the scalar kernels of a layer run there, next to the matrix-core kernels.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool ok = false;
};

qmoe_status side_stream(SideStream *out)
{
    static SideStream cached[64];
    static std::mutex mu;
    int dev = 0;
    QMOE_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return QMOE_E_LIMIT;
    std::lock_guard<std::mutex> lock(mu);
    SideStream &c = cached[dev];
    if (!c.ok) {
        QMOE_HIP_TRY(hipStreamCreateWithFlags(&c.stream, hipStreamNonBlocking));
        QMOE_HIP_TRY(hipEventCreateWithFlags(&c.fork, hipEventDisableTiming));
        QMOE_HIP_TRY(hipEventCreateWithFlags(&c.join, hipEventDisableTiming));
        c.ok = true;
    }
    *out = c;
    return QMOE_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct ProductPlan {
    int threads, rows_per_item, blocks_per_pass, tb_max, lds_dict_entries, grid;
    int stage_out;  // results of a block staged in LDS (first product of a layer, LDS permitting)
    int order_l2;   // device-order streams: the table is read from L2 instead of being staged in LDS
    size_t smem;
};

// Pick the token tile, workgroup size, blocks per matrix and grid for a product over rows x cols
// matrices with the lane-per-row kernel (compressed path).
qmoe_status plan_product(int rows, int cols, bool run_table, long long max_passes_hint, ProductPlan *p,
                         int n_order = 0, int force_blocks = 0, int stage_out_row_bytes = 0, bool minmax = false)
{
    DeviceInfo di;
    const qmoe_status st = device_info(&di);
    if (st != QMOE_OK) return st;
    const Tuning &tu = tuning();
    const size_t max_lds = (size_t)di.max_lds;
    const size_t fixed = 128;  // token ids, item hand-out
    // activations: bf16, 8 bytes per column for up to four tokens (one token uses the
    // {0,+x,0,-x} record), 16 bytes for eight
    auto xs_bytes = [&](int tb) { return (size_t)(cols + kPadCols) * 2 * (size_t)std::max(tb, 4); };
    if (xs_bytes(1) + fixed > max_lds) return QMOE_E_LIMIT;

    // Keep the leading run entries in LDS when the launch is long enough to pay for staging
    // them (one copy per workgroup): table reads that go to L2 cost a cycle per lane.
    const double codes_per_row = std::max(1.0, cols / 22.0);
    const double est_codes = (double)max_passes_hint * rows * codes_per_row;
    const bool lds_table = n_order == 0 && run_table && tu.lds_dict_entries >= 0 && max_lds >= 128 * 1024 &&
                           (tu.lds_dict_entries > 0 || est_codes / di.cus >= 1.0e6);
    // tiles of eight tokens cost more per token than two tiles of four (16-byte LDS gathers,
    // register pressure), so four is the default
    int tb = 4;
    // Device-order streams: the whole table goes to LDS and the tile takes what is left; only a
    // call whose activations leave no room for the table reads it from L2 (measured: that is
    // slower even for the smallest workload, where one 65 KB copy per workgroup looked like
    // the price to avoid: 0.126 against 0.102 ms).
    p->order_l2 = 0;
    if (n_order > 0) {
        const bool fits = xs_bytes(1) + fixed + 4 * (size_t)n_order + 16384 <= max_lds;
        if (tu.lds_dict_entries < 0 || !fits) {
            p->order_l2 = 1;
            n_order = 0;
        }
    }
    if (n_order > 0) {
        while (tb > 4 && xs_bytes(tb) + fixed + 4 * (size_t)n_order + 16384 > max_lds) tb >>= 1;
    } else if (p->order_l2) {
        while (tb > 4 && xs_bytes(tb) + fixed > max_lds / 2) tb >>= 1;
    } else if (lds_table) {
        while (tb > 4 && xs_bytes(tb) > 36 * 1024) tb >>= 1;
    } else {
        while (tb > 4 && xs_bytes(tb) + fixed > max_lds / 2) tb >>= 1;
    }
    if (tu.token_tile > 0) {
        tb = 1;
        while (tb * 2 <= tu.token_tile && tb < kMaxTokenTile) tb <<= 1;
    }
    while (tb > 4 && xs_bytes(tb) + fixed > max_lds) tb >>= 1;
    int lds_dict = n_order;
    if (lds_table) {
        const size_t room = (max_lds - xs_bytes(tb) - fixed) / 4;
        lds_dict = (int)std::min<size_t>(room, kTableEntries);
        if (tu.lds_dict_entries > 0) lds_dict = std::min(lds_dict, tu.lds_dict_entries);
        if (lds_dict < 4096) lds_dict = 0;
    }
    p->tb_max = tb;
    const int fit = (int)std::max<size_t>(1, max_lds / (xs_bytes(tb) + fixed + 4 * (size_t)lds_dict));

    // Lanes per matrix: a lane should own at least ~256 codewords (eight 64-byte chunks), and
    // rows / lanes should round up with little waste since a wavefront is as slow as its
    // lane with the most rows.  Search workgroup sizes and block counts for the best fill.
    const int want_rpl = std::max(1, (int)std::ceil(256.0 / codes_per_row));
    // 768 rather than 1024 lanes: measured 4 % faster on 6144-row matrices (12 wavefronts keep
    // the compute unit as busy as 16 do, and each gets more of the caches)
    const int max_threads = fit >= 4 ? 256 : (fit >= 2 ? 512 : 768);
    int best_t = 64, best_b = 1;
    double best_score = -1.0;
    for (int b = 1; b <= 64; b++) {
        if (force_blocks > 0 && b != std::min(force_blocks, 64)) continue;
        for (int t = 64; t <= max_threads; t += 64) {
            const long long nl = (long long)b * t;
            const int rpl = (int)((rows + nl - 1) / nl);
            if (rpl < want_rpl && force_blocks <= 0 && !(b == 1 && t == 64)) continue;
            const double fill = (double)rows / ((double)nl * rpl);
            // fill first, then larger workgroups (occupancy) and few blocks (less restaging)
            const double score = fill * (0.75 + 0.25 * (double)t / max_threads) - 0.002 * b;
            if (score > best_score) { best_score = score; best_t = t; best_b = b; }
        }
    }
    if (tu.threads > 0) {
        best_t = std::max(64, std::min(kProductMaxThreads, tu.threads / 64 * 64));
        const int rpl = tu.rows_per_item > 0 ? tu.rows_per_item : want_rpl;
        best_b = std::max(1, (int)((rows + (long long)best_t * rpl - 1) / ((long long)best_t * rpl)));
    }
    p->threads = best_t;
    p->blocks_per_pass = best_b;
    // most rows a block can own under the even split of rows over lanes
    const long long all_lanes = (long long)best_b * best_t;
    p->rows_per_item = (int)std::min<long long>(rows, (long long)best_t * (rows / all_lanes + 1));
    // binary16 scale, or bf16 (w_min, w_max) pair, of every row of a block
    const size_t scale_bytes = ((size_t)p->rows_per_item * (minmax ? 4 : 2) + 15) / 16 * 16;
    if (lds_dict > 0 && n_order == 0) {
        // the row scales take their share of LDS from the table
        const size_t room = max_lds - xs_bytes(tb) - fixed - scale_bytes;
        lds_dict = (int)std::min<size_t>((size_t)lds_dict, room / 4);
        if (lds_dict < 4096) lds_dict = 0;
    }
    p->lds_dict_entries = lds_dict;
    p->smem = xs_bytes(tb) + fixed + scale_bytes + 4 * (size_t)lds_dict;
    if (p->smem > max_lds) return QMOE_E_LIMIT;
    p->stage_out = 0;
    if (stage_out_row_bytes > 0) {
        // [tile][rows of a block, rounded up to 8] values after the table (itself rounded up to 16 bytes)
        const size_t table_end = xs_bytes(tb) + fixed + scale_bytes + ((4 * (size_t)lds_dict + 15) & ~(size_t)15);
        const size_t need = (size_t)tb * (((size_t)p->rows_per_item + 7) & ~(size_t)7) * stage_out_row_bytes;
        if (table_end + need <= max_lds) {
            p->stage_out = 1;
            p->smem = table_end + need;
        }
    }
    const int wg_per_cu = tu.grid_per_cu > 0 ? tu.grid_per_cu : std::max(1, std::min(fit, 2048 / best_t));
    long long grid = (long long)di.cus * wg_per_cu;
    const long long items = max_passes_hint * p->blocks_per_pass;
    if (items < grid) grid = std::max(1LL, items);
    p->grid = (int)grid;
    return QMOE_OK;
}

// A layer call with fewer work items than compute units (few tokens) splits every pass over
// a matrix between several workgroups; 0 = let plan_product choose (one block as a rule).
int layer_blocks_hint(int n_experts, int n_tokens)
{
    DeviceInfo di;
    if (device_info(&di) != QMOE_OK) return 0;
    // experts that receive a token under uniform routing, or tiles of four tokens if that is more
    const double active = n_experts * (1.0 - std::exp(-(double)n_tokens / n_experts));
    const int items = std::max(1, (int)std::max(active, n_tokens / 4.0));
    const int b = di.cus / items;
    return b >= 2 ? std::min(b, 8) : 0;
}

// The dense bf16 comparator keeps its own simple plan: token-major fp32 activations in
// LDS, one wavefront per row.
qmoe_status plan_dense(int rows, int cols, long long max_passes_hint, ProductPlan *p)
{
    DeviceInfo di;
    const qmoe_status st = device_info(&di);
    if (st != QMOE_OK) return st;
    const size_t max_lds = (size_t)di.max_lds;
    const size_t plane_bytes = (size_t)((cols + 3) / 4 * 4) * sizeof(float);
    int tb = kMaxTokenTile;
    while (tb > 1 && plane_bytes * tb + 128 > max_lds) tb >>= 1;
    if (plane_bytes * tb + 128 > max_lds) return QMOE_E_LIMIT;
    p->tb_max = tb;
    p->lds_dict_entries = 0;
    p->smem = plane_bytes * tb + 128;
    const int fit = (int)std::max<size_t>(1, max_lds / p->smem);
    p->threads = fit >= 2 ? 512 : 1024;
    p->rows_per_item = std::min(rows, 4 * (p->threads / 64));
    p->blocks_per_pass = (rows + p->rows_per_item - 1) / p->rows_per_item;
    long long grid = (long long)di.cus * std::max(1, std::min(fit, 2048 / p->threads));
    const long long items = max_passes_hint * p->blocks_per_pass;
    if (items < grid) grid = std::max(1LL, items);
    p->grid = (int)grid;
    return QMOE_OK;
}

template <typename K>
qmoe_status allow_lds(K kernel, size_t smem)
{
    if (smem > 48 * 1024)
        QMOE_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    return QMOE_OK;
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

template <int DICT, int EPI>
qmoe_status launch_product_as(const ProductArgs &a, const ProductPlan &p, hipStream_t s)
{
    return a.minmax ? launch_product_grid<DICT, EPI, 1>(a, p, s) : launch_product_grid<DICT, EPI, 0>(a, p, s);
}

qmoe_status launch_product(const ProductArgs &a, const ProductPlan &p, bool run, hipStream_t s)
{
    if (a.code_order && p.order_l2)
        return a.epilogue ? launch_product_as<kDictOrderL2, 1>(a, p, s) : launch_product_as<kDictOrderL2, 0>(a, p, s);
    if (a.code_order)
        return a.epilogue ? launch_product_as<kDictOrder, 1>(a, p, s) : launch_product_as<kDictOrder, 0>(a, p, s);
    if (!run) return a.epilogue ? launch_product_as<kDictWords, 1>(a, p, s) : launch_product_as<kDictWords, 0>(a, p, s);
    if (p.lds_dict_entries > 0)
        return a.epilogue ? launch_product_as<kDictRunLds, 1>(a, p, s) : launch_product_as<kDictRunLds, 0>(a, p, s);
    return a.epilogue ? launch_product_as<kDictRun, 1>(a, p, s) : launch_product_as<kDictRun, 0>(a, p, s);
}

// Which experts of a layer go to the matrix-core kernel, and its launch shape.
struct MmPlan {
    int min_tokens = 0x7FFFFFFF;  // experts with at least this many tokens; INT_MAX = path off
    int grid = 0;
    size_t smem = 0;
};

void mm_rows(int rows, int *row_blocks, int *rows_per_block)
{
    const int nb = (rows + kMmThreads - 1) / kMmThreads;
    const int per = (rows + nb - 1) / nb;
    *row_blocks = nb;
    *rows_per_block = std::min(kMmThreads, (per + 63) / 64 * 64);
}

qmoe_status plan_mm(const qmoe_dict *d, int code_order, int d_model, int d_ff, int n_tokens, bool x_aligned,
                    MmPlan *mp)
{
    *mp = MmPlan{};
    DeviceInfo di;
    const qmoe_status st = device_info(&di);
    if (st != QMOE_OK) return st;
    const Tuning &tu = tuning();
    const int n_order = (int)d->order_table.size();
    const bool fits = mm_lds_bytes(n_order) <= (size_t)di.max_lds;
    // 16-byte activation loads: widths divisible by eight, aligned base
    if (code_order != 1 || n_order == 0 || d->max_nonzeros > kRunMaxNonzeros || !fits || (d_model % 8) ||
        (d_ff % 8) || !x_aligned || tu.mfma_min_tokens < 0)
        return QMOE_OK;
    // A tile is walked column step by column step by one workgroup per 512 rows: a long chain
    // that pays only when the scalar kernel would need several rounds of items per compute
    // unit anyway.  With few tokens in the call (measured: 512 tokens on 128 experts) the
    // scalar kernel finishes every expert in one round and the chain would be the critical path.
    if (tu.mfma_min_tokens == 0 && n_tokens < 4 * di.cus) return QMOE_OK;
    mp->min_tokens = tu.mfma_min_tokens > 0 ? tu.mfma_min_tokens : kMmMinTokensDefault;
    mp->grid = di.cus;
    mp->smem = mm_lds_bytes(n_order);
    return QMOE_OK;
}

// rows_per_block: 0 = as few workgroups per matrix as possible (a layer call has many
// matrices); otherwise a multiple of 64 up to 512.
qmoe_status launch_product_mm(ProductArgs a, const MmPlan &mp, hipStream_t s, int rows_per_block = 0)
{
    if (rows_per_block > 0) {
        a.mm_rows_per_block = rows_per_block;
        a.mm_row_blocks = (a.rows + rows_per_block - 1) / rows_per_block;
    } else {
        mm_rows(a.rows, &a.mm_row_blocks, &a.mm_rows_per_block);
    }
    a.mm_stagger = tuning().mm_stagger > 0 ? 1 : 0;
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

qmoe_status check_matrix_args(const qmoe_dict *d, const qmoe_matrix *W)
{
    if (!d || !W) return QMOE_E_INVALID_ARG;
    if (!W->codes || !W->row_off || (!W->scale_f16 && !W->minmax_bf16) || W->rows < 1 || W->cols < 2 || (W->cols & 1))
        return QMOE_E_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(W->minmax_bf16) % 4) return QMOE_E_INVALID_ARG;  // pairs are read as one word
    if (W->cols > kMaxCols) return QMOE_E_LIMIT;
    if (!d->dev) return QMOE_E_NO_DEVICE_DICT;
    return QMOE_OK;
}

void fill_tables(const qmoe_dict *d, ProductArgs *a, int code_order)
{
    const unsigned char *base = static_cast<const unsigned char *>(d->dev);
    a->run = reinterpret_cast<const uint32_t *>(base + kDevRunOffset);
    a->words = reinterpret_cast<const uint32_t *>(base + kDevWordsOffset);
    a->order_table = reinterpret_cast<const uint32_t *>(base + kDevOrderTableOffset);
    a->n_groups = d->n_groups;
    a->n_order = (int)d->order_table.size();
    a->code_order = code_order;
}

// Splits a format argument (QMOE_FORMAT_* bits) into the numbering and the grid.
qmoe_status split_format(int format, int *code_order, bool *minmax)
{
    if (format < 0 || (format & ~(QMOE_FORMAT_DEVICE_ORDER | QMOE_FORMAT_GRID_MINMAX))) return QMOE_E_INVALID_ARG;
    *code_order = (format & QMOE_FORMAT_DEVICE_ORDER) ? 1 : 0;
    *minmax = (format & QMOE_FORMAT_GRID_MINMAX) != 0;
    return QMOE_OK;
}

qmoe_status check_code_order(const qmoe_dict *d, int code_order)
{
    if (code_order != 0 && code_order != 1) return QMOE_E_INVALID_ARG;
    if (code_order == 1 && d->order_table.empty()) return QMOE_E_LIMIT;
    return QMOE_OK;
}

qmoe_status layer_limits(int n_experts, int d_model, int d_ff, int n_tokens)
{
    if (n_experts < 1 || d_model < 2 || d_ff < 2 || n_tokens < 1 || (d_model & 1) || (d_ff & 1))
        return QMOE_E_INVALID_ARG;
    if (n_experts > kMaxExperts || n_tokens > kMaxTokens || d_model > kMaxCols || d_ff > kMaxCols)
        return QMOE_E_LIMIT;
    return QMOE_OK;
}

struct LayerPtrs {
    int *tok_off, *perm, *counters;
    Item *items_wi, *items_wo, *items_mm;
    uint16_t *hidden;
};

LayerPtrs layer_ptrs(void *ws, const qmoe_ws_layout &l)
{
    unsigned char *b = static_cast<unsigned char *>(ws);
    return LayerPtrs{reinterpret_cast<int *>(b + l.tok_off), reinterpret_cast<int *>(b + l.perm),
                     reinterpret_cast<int *>(b + l.counters), reinterpret_cast<Item *>(b + l.items_wi),
                     reinterpret_cast<Item *>(b + l.items_wo), reinterpret_cast<Item *>(b + l.items_mm),
                     reinterpret_cast<uint16_t *>(b + l.hidden)};
}

qmoe_status launch_dispatch(const int32_t *expert_idx, int n_tokens, int n_experts, int d_model,
                            const LayerPtrs &lp, int tb_wi, int tb_wo, int mm_min, float *y, hipStream_t s)
{
    DispatchArgs da;
    da.expert_idx = expert_idx;
    da.n_tokens = n_tokens;
    da.n_experts = n_experts;
    da.tok_off = lp.tok_off;
    da.perm = lp.perm;
    da.counters = lp.counters;
    da.items_wi = lp.items_wi;
    da.items_wo = lp.items_wo;
    da.items_mm = lp.items_mm;
    da.tb_wi = tb_wi;
    da.tb_wo = tb_wo;
    da.mm_min = mm_min;
    da.y = y;
    da.d_model = d_model;
    // token counts, scan scratch (17 x 12, rounded up), two arrays of one round of tokens
    const size_t smem = sizeof(int) * ((size_t)n_experts + 256 + 2 * 1024);
    const qmoe_status st = allow_lds(k_dispatch, smem);
    if (st != QMOE_OK) return st;
    hipLaunchKernelGGL(k_dispatch, dim3(1), dim3(1024), smem, s, da);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

}  // namespace
}  // namespace qmoe

using namespace qmoe;

extern "C" {

int qmoe_last_hip_error(void) { return g_last_hip_error.load(); }

qmoe_status qmoe_dict_upload(qmoe_dict *d, void *dev_buf, size_t dev_bytes, void *stream)
{
    if (!d || !dev_buf) return QMOE_E_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dev_buf) % 256) return QMOE_E_INVALID_ARG;
    if (dev_bytes < kDevDictBytes) return QMOE_E_BUFFER_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned char *b = static_cast<unsigned char *>(dev_buf);
    QMOE_HIP_TRY(hipMemcpyAsync(b + kDevRunOffset, d->run.data(), sizeof(uint32_t) * kTableEntries,
                                hipMemcpyHostToDevice, s));
    QMOE_HIP_TRY(hipMemcpyAsync(b + kDevWordsOffset, d->words.data(), 2 * sizeof(uint32_t) * kTableEntries,
                                hipMemcpyHostToDevice, s));
    if (!d->order_table.empty()) {
        QMOE_HIP_TRY(hipMemcpyAsync(b + kDevOrderTableOffset, d->order_table.data(),
                                    sizeof(uint32_t) * d->order_table.size(), hipMemcpyHostToDevice, s));
        QMOE_HIP_TRY(hipMemcpyAsync(b + kDevOrderMapOffset, d->order_map.data(), sizeof(uint16_t) * kTableEntries,
                                    hipMemcpyHostToDevice, s));
    }
    if (!d->code.empty() && d->code.size() <= (size_t)kMaxTrieNodes) {
        QMOE_HIP_TRY(hipMemcpyAsync(b + kDevTrieChildOffset, d->child.data(), sizeof(int32_t) * d->child.size(),
                                    hipMemcpyHostToDevice, s));
        QMOE_HIP_TRY(hipMemcpyAsync(b + kDevTrieCodeOffset, d->code.data(), sizeof(int32_t) * d->code.size(),
                                    hipMemcpyHostToDevice, s));
    }
    d->dev = dev_buf;
    return QMOE_OK;
}

qmoe_status qmoe_encode_device(const qmoe_dict *d, const int8_t *ternary, int rows, int cols, uint16_t *codes,
                               size_t codes_cap, uint32_t *row_off, int32_t *status, void *stream)
{
    if (!d || !ternary || !codes || !row_off || !status || rows < 1 || cols < 2 || (cols & 1)) return QMOE_E_INVALID_ARG;
    if (!d->dev) return QMOE_E_NO_DEVICE_DICT;
    if (d->code.empty() || d->code.size() > (size_t)kMaxTrieNodes) return QMOE_E_LIMIT;
    const unsigned char *base = static_cast<const unsigned char *>(d->dev);
    EncodeArgs a{};
    a.tern = ternary;
    a.rows = rows;
    a.cols = cols;
    a.child = reinterpret_cast<const int32_t *>(base + kDevTrieChildOffset);
    a.code = reinterpret_cast<const int32_t *>(base + kDevTrieCodeOffset);
    a.row_off = row_off;
    a.codes = codes;
    a.codes_cap = codes_cap;
    a.status = status;
    hipStream_t s = static_cast<hipStream_t>(stream);
    QMOE_HIP_TRY(hipMemsetAsync(status, 0, 2 * sizeof(int32_t), s));
    const int grid = (rows + 255) / 256;
    hipLaunchKernelGGL(k_encode<false>, dim3(grid), dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_encode_offsets, dim3(1), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(k_encode<true>, dim3(grid), dim3(256), 0, s, a);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

qmoe_status qmoe_decode_matvec(const qmoe_dict *d, const qmoe_matrix *W, const uint16_t *x_bf16, int batch,
                               float *y, void *stream)
{
    qmoe_status st = check_matrix_args(d, W);
    if (st != QMOE_OK) return st;
    if (!x_bf16 || !y || batch < 1) return QMOE_E_INVALID_ARG;
    const int code_order = (int)W->code_order;
    if ((st = check_code_order(d, code_order)) != QMOE_OK) return st;
    const bool run = d->max_nonzeros <= kRunMaxNonzeros;
    DeviceInfo di;
    if ((st = device_info(&di)) != QMOE_OK) return st;
    // activations of a tile in LDS: 8 bytes per column for up to four tokens, 16 for eight
    int tb = batch > 4 ? 8 : 4;
    auto xs_bytes = [&](int t) { return (size_t)(W->cols + kPadCols) * 2 * (size_t)t; };
    if (tb == 8 && xs_bytes(8) > (size_t)di.max_lds) tb = 4;
    if (xs_bytes(tb) > (size_t)di.max_lds) return QMOE_E_LIMIT;
    if (tuning().token_tile > 0) tb = std::max(1, std::min(tb, tuning().token_tile));
    ProductArgs a{};
    a.mats = nullptr;
    a.single = *W;
    fill_tables(d, &a, code_order);
    a.n_experts = 1;
    a.batch = batch;
    a.x = x_bf16;
    a.x_by_slot = 1;
    a.ldx = W->cols;
    a.out = y;
    a.ld_out = W->rows;
    a.rows = W->rows;
    a.cols = W->cols;
    a.tb_max = tb;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Many tokens: the matrix-core kernel decodes the matrix once per 64 tokens instead of once
    // per 8.  One matrix has few row blocks of 512, so the blocks are made as small as they can
    // be with all of them resident at once (every block still decodes only its own rows; a
    // block's time is set by the length of a row, not by how many rows it has).
    {
        const Tuning &tu = tuning();
        const int n_order = (int)d->order_table.size();
        if (code_order == 1 && run && n_order > 0 && tu.mfma_min_tokens >= 0 && W->cols % 8 == 0 &&
            reinterpret_cast<uintptr_t>(x_bf16) % 16 == 0 && mm_lds_bytes(n_order) <= (size_t)di.max_lds) {
            const int tiles = (batch + kMmTokens - 1) / kMmTokens;
            int rpb = 64;
            while (rpb < kMmThreads && (long long)tiles * ((W->rows + rpb - 1) / rpb) > di.cus) rpb += 64;
            const long long blocks = (long long)tiles * ((W->rows + rpb - 1) / rpb);
            // Measured on this GPU (microseconds): a round of the matrix-core kernel takes about
            // 8 + 0.0225 per column; the other kernel works through tiles of eight tokens at 0.62
            // million weights per microsecond with one workgroup resident per compute unit (long
            // rows: the tile's activations fill the LDS), 1.6 with four, 2.5-3 with eight.
            const double rounds = std::ceil((double)blocks / di.cus);
            const double t_mm = rounds * (8.0 + 0.0225 * W->cols);
            const int resident = (int)std::max<size_t>(1, std::min<size_t>(8, (size_t)di.max_lds / xs_bytes(8)));
            const double rate = 0.62e6 * (1.0 + 0.55 * (resident - 1));
            const double t_rows = std::max(8.5, 4.0 + std::ceil(batch / 8.0) * (double)W->rows * W->cols / rate);
            const bool take = tu.mfma_min_tokens > 0 ? batch >= tu.mfma_min_tokens : t_mm < t_rows;
            if (take) {
                a.minmax = W->minmax_bf16 ? 1 : 0;
                a.epilogue = 0;
                MmPlan mp;
                mp.smem = mm_lds_bytes(n_order);
                mp.grid = (int)std::min<long long>(blocks, di.cus);
                return launch_product_mm(a, mp, s, rpb);
            }
        }
    }
    const int threads = 256;  // 16 rows at a time
    const long long items = (long long)((batch + tb - 1) / tb) * ((W->rows + threads / 16 - 1) / (threads / 16));
    const int grid = (int)std::min<long long>(items, 8LL * di.cus);
    const size_t smem = xs_bytes(std::max(tb, 4));
    auto launch = [&](auto kernel) -> qmoe_status {
        const qmoe_status lst = allow_lds(kernel, smem);
        if (lst != QMOE_OK) return lst;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), smem, s, a);
        return QMOE_OK;
    };
    if (W->minmax_bf16)
        st = run ? launch(k_matvec_rows<true, 1>) : launch(k_matvec_rows<false, 1>);
    else
        st = run ? launch(k_matvec_rows<true, 0>) : launch(k_matvec_rows<false, 0>);
    if (st != QMOE_OK) return st;
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

qmoe_status qmoe_decode_dense(const qmoe_dict *d, const qmoe_matrix *W, int8_t *out, int path, void *stream)
{
    qmoe_status st = check_matrix_args(d, W);
    if (st != QMOE_OK) return st;
    if (!out || (path != 0 && path != 1)) return QMOE_E_INVALID_ARG;
    const int code_order = (int)W->code_order;
    if ((st = check_code_order(d, code_order)) != QMOE_OK) return st;
    if (code_order && path == 1) return QMOE_E_INVALID_ARG;  // device-order codes do not index the interchange table
    const bool run = path == 0 && d->max_nonzeros <= kRunMaxNonzeros;
    ProductArgs a{};
    a.single = *W;
    fill_tables(d, &a, code_order);
    a.rows = W->rows;
    a.cols = W->cols;
    a.lds_dict_entries = 0;
    DeviceInfo di;
    if ((st = device_info(&di)) != QMOE_OK) return st;
    const int groups = 256 / 16;
    const int grid = std::max(1, std::min((W->rows + groups - 1) / groups, di.cus * 8));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (run)
        hipLaunchKernelGGL(k_decode_dense<true>, dim3(grid), dim3(256), 0, s, a, out);
    else
        hipLaunchKernelGGL(k_decode_dense<false>, dim3(grid), dim3(256), 0, s, a, out);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

qmoe_status qmoe_decompress(const qmoe_dict *d, const qmoe_matrix *mats, int code_order, int n_mats, int rows,
                            int cols, int out_kind, void *const *out, void *stream)
{
    bool minmax = false;
    {
        const qmoe_status fst = split_format(code_order, &code_order, &minmax);
        if (fst != QMOE_OK) return fst;
    }
    if (!d || !mats || !out || n_mats < 1 || rows < 1 || cols < 2 || (out_kind != 0 && out_kind != 1))
        return QMOE_E_INVALID_ARG;
    if (cols % 8) return QMOE_E_INVALID_ARG;  // whole 8-column stores
    if (cols > kMaxCols) return QMOE_E_LIMIT;
    if (!d->dev) return QMOE_E_NO_DEVICE_DICT;
    if (code_order != 1) return QMOE_E_INVALID_ARG;  // the ring decoder reads the device-order table from LDS
    qmoe_status st = check_code_order(d, code_order);
    if (st != QMOE_OK) return st;
    if (d->max_nonzeros > kRunMaxNonzeros) return QMOE_E_LIMIT;
    DeviceInfo di;
    if ((st = device_info(&di)) != QMOE_OK) return st;
    DecompressArgs a{};
    a.mats = mats;
    a.out = out;
    a.n_mats = n_mats;
    a.rows = rows;
    a.cols = cols;
    mm_rows(rows, &a.row_blocks, &a.rows_per_block);
    a.order_table = reinterpret_cast<const uint32_t *>(static_cast<const unsigned char *>(d->dev) + kDevOrderTableOffset);
    a.n_groups = d->n_groups;
    a.n_order = (int)d->order_table.size();
    const size_t smem = (((size_t)a.n_order * 4 + 15) & ~(size_t)15) + (size_t)kMmThreads * kMmWRowBytes;
    if (smem > (size_t)di.max_lds) return QMOE_E_LIMIT;
    const long long total = (long long)n_mats * a.row_blocks;
    const int grid = (int)std::min<long long>(total, 2LL * di.cus);
    hipStream_t s = static_cast<hipStream_t>(stream);
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

qmoe_status qmoe_moe_layer_ws_layout(int n_experts, int d_model, int d_ff, int n_tokens, qmoe_ws_layout *out)
{
    if (!out) return QMOE_E_INVALID_ARG;
    const qmoe_status st = layer_limits(n_experts, d_model, d_ff, n_tokens);
    if (st != QMOE_OK) return st;
    size_t off = 0;
    out->tok_off = off;  off = align_up(off + sizeof(int) * ((size_t)n_experts + 1), 256);
    out->perm = off;     off = align_up(off + sizeof(int) * (size_t)n_tokens, 256);
    out->counters = off; off = align_up(off + sizeof(int) * kLayerCounters, 256);
    out->items_wi = off; off = align_up(off + sizeof(Item) * (size_t)n_tokens, 256);
    out->items_wo = off; off = align_up(off + sizeof(Item) * (size_t)n_tokens, 256);
    out->items_mm = off; off = align_up(off + sizeof(Item) * (size_t)n_tokens, 256);
    out->hidden = off;   off = align_up(off + sizeof(uint16_t) * (size_t)n_tokens * (size_t)d_ff, 256);
    out->total = off;
    return QMOE_OK;
}

size_t qmoe_moe_layer_workspace(int n_experts, int d_model, int d_ff, int n_tokens)
{
    qmoe_ws_layout l;
    return qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens, &l) == QMOE_OK ? l.total : 0;
}

qmoe_status qmoe_moe_dispatch(const qmoe_dict *d, int code_order, const int32_t *expert_idx, int n_tokens,
                              int n_experts, int d_model, int d_ff, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    qmoe_ws_layout l;
    qmoe_status st = qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens, &l);
    if (st != QMOE_OK) return st;
    if (!d || !expert_idx) return QMOE_E_INVALID_ARG;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < l.total)
        return QMOE_E_WORKSPACE;
    bool minmax = false;
    if ((st = split_format(code_order, &code_order, &minmax)) != QMOE_OK) return st;
    if ((st = check_code_order(d, code_order)) != QMOE_OK) return st;
    const bool run = d->max_nonzeros <= kRunMaxNonzeros;
    const int n_order = code_order ? (int)d->order_table.size() : 0;
    ProductPlan pwi, pwo;
    MmPlan mp;
    const int spread = layer_blocks_hint(n_experts, n_tokens);
    if ((st = plan_product(d_ff, d_model, run, n_tokens, &pwi, n_order,
                           tuning().blocks_first > 0 ? tuning().blocks_first : spread,
                           (d_ff % 8 == 0 && tuning().stage_out >= 0) ? 2 : 0, minmax)) != QMOE_OK)
        return st;
    if ((st = plan_product(d_model, d_ff, run, n_tokens, &pwo, n_order,
                           tuning().blocks_second > 0 ? tuning().blocks_second : spread,
                           (d_model % 8 == 0 && tuning().stage_out >= 0) ? 4 : 0, minmax)) != QMOE_OK)
        return st;
    if ((st = plan_mm(d, code_order, d_model, d_ff, n_tokens, true, &mp)) != QMOE_OK) return st;
    return launch_dispatch(expert_idx, n_tokens, n_experts, d_model, layer_ptrs(workspace, l), pwi.tb_max,
                           pwo.tb_max, mp.min_tokens, nullptr, static_cast<hipStream_t>(stream));
}

qmoe_status qmoe_moe_layer_forward(const qmoe_dict *d, const qmoe_matrix *wi, const qmoe_matrix *wo,
                                   int code_order, int n_experts, int d_model, int d_ff, const uint16_t *x_bf16,
                                   const int32_t *expert_idx, const float *gate, int n_tokens, float *y,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    qmoe_ws_layout l;
    qmoe_status st = qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens, &l);
    if (st != QMOE_OK) return st;
    if (!d || !wi || !wo || !x_bf16 || !expert_idx || !y) return QMOE_E_INVALID_ARG;
    if (!d->dev) return QMOE_E_NO_DEVICE_DICT;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < l.total)
        return QMOE_E_WORKSPACE;
    bool minmax = false;
    if ((st = split_format(code_order, &code_order, &minmax)) != QMOE_OK) return st;
    if ((st = check_code_order(d, code_order)) != QMOE_OK) return st;
    const bool run = d->max_nonzeros <= kRunMaxNonzeros;
    const int n_order = code_order ? (int)d->order_table.size() : 0;
    ProductPlan pwi, pwo;
    const int spread = layer_blocks_hint(n_experts, n_tokens);
    if ((st = plan_product(d_ff, d_model, run, n_tokens, &pwi, n_order,
                           tuning().blocks_first > 0 ? tuning().blocks_first : spread,
                           (d_ff % 8 == 0 && tuning().stage_out >= 0) ? 2 : 0, minmax)) != QMOE_OK)
        return st;
    if ((st = plan_product(d_model, d_ff, run, n_tokens, &pwo, n_order,
                           tuning().blocks_second > 0 ? tuning().blocks_second : spread,
                           (d_model % 8 == 0 && tuning().stage_out >= 0) ? 4 : 0, minmax)) != QMOE_OK)
        return st;
    MmPlan mp;
    if ((st = plan_mm(d, code_order, d_model, d_ff, n_tokens, reinterpret_cast<uintptr_t>(x_bf16) % 16 == 0, &mp)) != QMOE_OK)
        return st;
    const bool mm = mp.min_tokens <= n_tokens;  // otherwise no expert can reach the threshold
    hipStream_t s = static_cast<hipStream_t>(stream);
    const LayerPtrs lp = layer_ptrs(workspace, l);
    const int phases = tuning().phases > 0 ? tuning().phases : 31;
    if (phases & 1)
        if ((st = launch_dispatch(expert_idx, n_tokens, n_experts, d_model, lp, pwi.tb_max, pwo.tb_max,
                                  mp.min_tokens, y, s)) != QMOE_OK)
            return st;

    // The experts with few tokens and the crowded ones are two independent chains of two
    // kernels (each second product reads only the hidden rows its own first product wrote).
    // With both kinds present the scalar chain goes to a side stream that forks from
    // `stream` after the dispatch and joins it again at the end, so the kernels fill each
    // other's idle compute units; the caller sees the usual stream order.
    const bool overlap = mm && tuning().overlap >= 0 && (phases & 6) && (phases & 24);
    hipStream_t s_scalar = s;
    SideStream side;
    if (overlap) {
        if ((st = side_stream(&side)) != QMOE_OK) return st;
        s_scalar = side.stream;
        QMOE_HIP_TRY(hipEventRecord(side.fork, s));
        QMOE_HIP_TRY(hipStreamWaitEvent(s_scalar, side.fork, 0));
    }
    ProductArgs a{};
    fill_tables(d, &a, code_order);
    a.n_experts = n_experts;
    a.max_items = n_tokens;
    a.perm = lp.perm;
    a.minmax = minmax ? 1 : 0;
    // first product: hidden[slot] = bf16(relu(Wi x[token]))
    ProductArgs a1 = a;
    a1.gate = nullptr;
    a1.mats = wi;
    a1.x = x_bf16;
    a1.x_by_slot = 0;
    a1.ldx = d_model;
    a1.out = lp.hidden;
    a1.ld_out = d_ff;
    a1.epilogue = 1;
    a1.rows = d_ff;
    a1.cols = d_model;
    // second product: y[token] = gate * Wo hidden[slot]
    ProductArgs a2 = a;
    a2.gate = gate;
    a2.mats = wo;
    a2.x = lp.hidden;
    a2.x_by_slot = 1;
    a2.ldx = d_ff;
    a2.out = y;
    a2.ld_out = d_model;
    a2.epilogue = 0;
    a2.rows = d_model;
    a2.cols = d_ff;
    // crowded experts (matrix cores) on `stream`: their tiles are the long items
    if (mm) {
        ProductArgs am = a1;
        am.items = lp.items_mm;
        am.n_items_dev = lp.counters + 7;
        am.work_counter = lp.counters + 8;
        if (phases & 8)
            if ((st = launch_product_mm(am, mp, s)) != QMOE_OK) return st;
        am = a2;
        am.items = lp.items_mm;
        am.n_items_dev = lp.counters + 7;
        am.work_counter = lp.counters + 9;
        if (phases & 16)
            if ((st = launch_product_mm(am, mp, s)) != QMOE_OK) return st;
    }
    // experts with few tokens (scalar kernels)
    a1.items = lp.items_wi;
    a1.n_items_dev = lp.counters + 3;
    a1.rows_per_item = pwi.rows_per_item;
    a1.blocks_per_pass = pwi.blocks_per_pass;
    a1.tb_max = pwi.tb_max;
    a1.lds_dict_entries = pwi.lds_dict_entries;
    a1.stage_out = pwi.stage_out;
    a1.work_counter = lp.counters + 5;
    if (phases & 2)
        if ((st = launch_product(a1, pwi, run, s_scalar)) != QMOE_OK) return st;
    a2.items = lp.items_wo;
    a2.n_items_dev = lp.counters + 4;
    a2.rows_per_item = pwo.rows_per_item;
    a2.blocks_per_pass = pwo.blocks_per_pass;
    a2.tb_max = pwo.tb_max;
    a2.lds_dict_entries = pwo.lds_dict_entries;
    a2.stage_out = pwo.stage_out && reinterpret_cast<uintptr_t>(y) % 16 == 0;
    a2.work_counter = lp.counters + 6;
    if (phases & 4)
        if ((st = launch_product(a2, pwo, run, s_scalar)) != QMOE_OK) return st;
    if (overlap) {
        QMOE_HIP_TRY(hipEventRecord(side.join, s_scalar));
        QMOE_HIP_TRY(hipStreamWaitEvent(s, side.join, 0));
    }
    return QMOE_OK;
}

qmoe_status qmoe_bf16_layer_forward(const uint16_t *const *wi_dense, const uint16_t *const *wo_dense,
                                    int n_experts, int d_model, int d_ff, const uint16_t *x_bf16,
                                    const int32_t *expert_idx, const float *gate, int n_tokens, float *y,
                                    void *workspace, size_t workspace_bytes, void *stream)
{
    qmoe_ws_layout l;
    qmoe_status st = qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens, &l);
    if (st != QMOE_OK) return st;
    if (!wi_dense || !wo_dense || !x_bf16 || !expert_idx || !y) return QMOE_E_INVALID_ARG;
    if ((d_model % 8) || (d_ff % 8)) return QMOE_E_INVALID_ARG;  // 16-byte row loads
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < l.total)
        return QMOE_E_WORKSPACE;
    ProductPlan pwi, pwo;
    if ((st = plan_dense(d_ff, d_model, n_tokens, &pwi)) != QMOE_OK) return st;
    if ((st = plan_dense(d_model, d_ff, n_tokens, &pwo)) != QMOE_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const LayerPtrs lp = layer_ptrs(workspace, l);
    const int phases = tuning().phases > 0 ? tuning().phases : 7;
    if (phases & 1)
        if ((st = launch_dispatch(expert_idx, n_tokens, n_experts, d_model, lp, pwi.tb_max, pwo.tb_max,
                                  0x7FFFFFFF, y, s)) != QMOE_OK)
            return st;
    DenseArgs a{};
    a.n_experts = n_experts;
    a.max_items = n_tokens;
    a.perm = lp.perm;
    a.mats = wi_dense;
    a.items = lp.items_wi;
    a.n_items_dev = lp.counters + 3;
    a.x = x_bf16;
    a.x_by_slot = 0;
    a.ldx = d_model;
    a.out = lp.hidden;
    a.ld_out = d_ff;
    a.gate = nullptr;
    a.epilogue = 1;
    a.rows = d_ff;
    a.cols = d_model;
    a.rows_per_item = pwi.rows_per_item;
    a.blocks_per_pass = pwi.blocks_per_pass;
    a.tb_max = pwi.tb_max;
    a.work_counter = lp.counters + 5;
    if (phases & 2) {
        if ((st = allow_lds(k_dense_bf16, pwi.smem)) != QMOE_OK) return st;
        hipLaunchKernelGGL(k_dense_bf16, dim3(pwi.grid), dim3(pwi.threads), pwi.smem, s, a);
        QMOE_HIP_TRY(hipGetLastError());
    }
    a.mats = wo_dense;
    a.items = lp.items_wo;
    a.n_items_dev = lp.counters + 4;
    a.x = lp.hidden;
    a.x_by_slot = 1;
    a.ldx = d_ff;
    a.out = y;
    a.ld_out = d_model;
    a.gate = gate;
    a.epilogue = 0;
    a.rows = d_model;
    a.cols = d_ff;
    a.rows_per_item = pwo.rows_per_item;
    a.blocks_per_pass = pwo.blocks_per_pass;
    a.tb_max = pwo.tb_max;
    a.work_counter = lp.counters + 6;
    if (phases & 4) {
        if ((st = allow_lds(k_dense_bf16, pwo.smem)) != QMOE_OK) return st;
        hipLaunchKernelGGL(k_dense_bf16, dim3(pwo.grid), dim3(pwo.threads), pwo.smem, s, a);
        QMOE_HIP_TRY(hipGetLastError());
    }
    return QMOE_OK;
}

qmoe_status qmoe_codes_to_device_order(const qmoe_dict *d, uint16_t *codes, size_t n_codes, void *stream)
{
    if (!d || !codes || n_codes == 0) return QMOE_E_INVALID_ARG;
    if (!d->dev) return QMOE_E_NO_DEVICE_DICT;
    if (d->order_table.empty()) return QMOE_E_LIMIT;
    DeviceInfo di;
    const qmoe_status st = device_info(&di);
    if (st != QMOE_OK) return st;
    const int grid = (int)std::min<size_t>((n_codes + 255) / 256, (size_t)di.cus * 32);
    const uint16_t *map = reinterpret_cast<const uint16_t *>(static_cast<const unsigned char *>(d->dev) +
                                                             kDevOrderMapOffset);
    hipLaunchKernelGGL(k_renumber, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), codes, n_codes, map);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

qmoe_status qmoe_stream_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || bytes == 0 || (bytes % 16) || reinterpret_cast<uintptr_t>(dst) % 16 ||
        reinterpret_cast<uintptr_t>(src) % 16)
        return QMOE_E_INVALID_ARG;
    DeviceInfo di;
    const qmoe_status st = device_info(&di);
    if (st != QMOE_OK) return st;
    const size_t n16 = bytes / 16;
    const int grid = (int)std::min<size_t>((n16 + 255) / 256, (size_t)di.cus * 32);
    hipLaunchKernelGGL(k_stream_copy, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n16);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

}  // extern "C"
