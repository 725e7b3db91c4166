// Shared by the HIP translation units of the library: argument blocks of the kernels, the
// device helpers several kernels use (table look-ups, activation staging, the gather form of
// a codeword's contribution) and the host-side launch functions each unit exports.
// Section 4.3.3 of the paper defines what the kernels compute; the mapping onto gfx950
// (CDNA4, wave64) is this library's own and is described where each kernel is defined:
//   qmoe_product.h / qmoe_product_*.hip  fused decode + product, a lane per row range
//   qmoe_product_mm.hip                  decode once, multiply on the matrix cores; decompression
//   qmoe_matvec.hip                      one matrix, a few tokens: 16 lanes per row; decode-only hook
//   qmoe_dispatch.hip                    tokens grouped by expert, work lists
//   qmoe_misc.hip                        device encoder, bf16 comparator, copy, renumbering
//   qmoe_api.hip                         launch planning and the C ABI
// Not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdio>
#include <type_traits>

#include "qmoe_internal.h"

namespace qmoe {

extern std::atomic<int> g_last_hip_error;  // defined in qmoe_api.hip

inline bool hip_failed(hipError_t e)
{
    if (e == hipSuccess) return false;
    g_last_hip_error.store((int)e);
    return true;
}
#define QMOE_HIP_TRY(expr)                           \
    do {                                             \
        if (::qmoe::hip_failed(expr)) return QMOE_E_HIP;     \
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
    int mm_row_blocks;  // matrix-core kernel: blocks of 64 rows per matrix (a wavefront's unit of work)
    int mm_in_step;     // matrix-core kernel: a workgroup's wavefronts may take eight consecutive units at a time, together
    int minmax;               // rows on the grid {w_min, 0, w_max} (host side: which kernel to launch)
    // matrix-core kernel, layer calls: the hidden vectors of a tile are kept in blocks of 16 tokens,
    // [8-column group][token of the block][8 columns] (a partial last block: its own token count),
    // in the same bytes the plain [slot][column] rows would take, so that the 16-byte operand
    // loads of the second product are consecutive over the 64 lanes of a wavefront
    int x_tiled, out_tiled;
};


struct DecompressArgs {
    const qmoe_matrix *mats;  // device array
    void *const *out;         // device array of destinations (row-major rows x cols), nullptr = skip
    int n_mats, rows, cols;
    int rows_per_block, row_blocks;
    const uint32_t *order_table;
    int n_groups, n_order;
};

struct DispatchArgs {
    const int *expert_idx;
    int n_tokens, n_experts;
    int *tok_off;   // [E+1]
    int *perm;      // [T]
    int *counters;  // [kLayerCounters]
    Item *items_wi, *items_wo, *items_mm;
    int tb_wi, tb_wo;
    int mm_min;     // experts with at least this many tokens go to the matrix-core kernel (tiles of 64)
    float *y;       // rows of dropped tokens are zeroed (may be nullptr)
    int d_model;
};

struct EncodeArgs {
    const int8_t *tern;   // [rows][cols], values -1 / 0 / +1
    int rows, cols;
    const int32_t *child, *code;
    uint32_t *row_off;    // [rows+1]
    uint16_t *codes;
    unsigned long long codes_cap;
    int *status;          // [2]: first error (qmoe_status, 0 = none), a row it happened in
};

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

struct DeviceInfo {
    int cus = 0;
    int max_lds = 0;
    bool ok = false;
};

struct ProductPlan {
    int threads, rows_per_item, blocks_per_pass, tb_max, lds_dict_entries, grid;
    int stage_out;  // results of a block staged in LDS (first product of a layer, LDS permitting)
    int order_l2;   // device-order streams: the table is read from L2 instead of being staged in LDS
    size_t smem;
};

// Which experts of a layer go to the matrix-core kernel, and its launch shape.
struct MmPlan {
    int min_tokens = 0x7FFFFFFF;  // experts with at least this many tokens; INT_MAX = path off
    int grid = 0;
    size_t smem = 0;
};

// matrix-core kernel: shape constants the planner needs
constexpr int kProductMaxThreads = 768;  // largest workgroup of k_product
constexpr int kMmThreads = 512;
constexpr int kMmTokens = 64;                  // tokens per tile
constexpr int kMmMinTokensDefault = 8;         // experts with fewer tokens stay on the scalar kernel

// ---------------------------------------------------------------- launch functions (one per kernel family)
// Each enqueues on `s` and returns QMOE_OK or QMOE_E_HIP; the callers have checked the arguments.
qmoe_status allow_lds_bytes(const void *kernel, size_t smem);
template <typename K>
inline qmoe_status allow_lds(K kernel, size_t smem)
{
    return allow_lds_bytes(reinterpret_cast<const void *>(kernel), smem);
}
qmoe_status launch_product(const ProductArgs &a, const ProductPlan &p, bool run, hipStream_t s);   // qmoe_product_*.hip
qmoe_status launch_product_sym(const ProductArgs &a, const ProductPlan &p, bool run, hipStream_t s);
qmoe_status launch_product_asym(const ProductArgs &a, const ProductPlan &p, bool run, hipStream_t s);
size_t mm_lds_bytes(int n_order);                                                                   // qmoe_product_mm.hip
qmoe_status launch_product_mm(ProductArgs a, const MmPlan &mp, hipStream_t s);
void mm_rows(int rows, int *row_blocks, int *rows_per_block);
qmoe_status launch_decompress(const DecompressArgs &a, int out_kind, bool minmax, int grid, size_t smem, hipStream_t s);
size_t decompress_lds_bytes(int n_order, int n_mats);  // table, rings, windows, one bit per matrix
qmoe_status launch_matvec_rows(const ProductArgs &a, bool run, bool minmax, int grid, int threads, size_t smem,
                               hipStream_t s);                                                      // qmoe_matvec.hip
qmoe_status launch_decode_dense(const ProductArgs &a, bool run, int8_t *out, int grid, hipStream_t s);
qmoe_status launch_dispatch_kernel(const DispatchArgs &da, hipStream_t s);                          // qmoe_dispatch.hip
qmoe_status launch_encode(const EncodeArgs &a, hipStream_t s);                                      // qmoe_misc.hip
qmoe_status launch_dense_bf16(const DenseArgs &a, const ProductPlan &p, hipStream_t s);
qmoe_status launch_stream_copy(void *dst, const void *src, size_t n16, int grid, hipStream_t s);
qmoe_status launch_renumber(uint16_t *codes, size_t n, const uint16_t *map, int grid, hipStream_t s);

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
// Where one row's codewords sit, for the kernels that give a lane one row: `pp` is the address
// of the 16-byte piece that holds the row's first codeword, `sub` that codeword's index in the
// piece (0..7), `left` the number of codewords, `last` the address of the piece that holds the
// last one, `pstride` the distance from a piece to the next of the same stream (16 with rows
// back to back; 1024 in the lane-interleaved layout, where the row is a part of the stream of
// the lane that owns it under the even split of rows over M.lanes lanes).  A row that is not
// live, or has no codewords, points at the matrix's first piece with left = 0.
struct RowStream {
    uintptr_t pp, last, pstride;
    uint32_t left, sub;
};

__device__ __forceinline__ RowStream row_stream(const qmoe_matrix &M, int row, bool live)
{
    RowStream r;
    r.pp = reinterpret_cast<uintptr_t>(M.codes);
    r.last = r.pp;
    r.pstride = M.lanes ? 1024u : 16u;
    r.left = 0u;
    r.sub = 0u;
    if (!live) return r;
    gp_u32 row_off = (gp_u32)M.row_off;
    const uint32_t cap = min(M.n_codes, kMaxCodes);
    const uint32_t K1 = min(row_off[row + 1], cap);
    const uint32_t K0 = min(row_off[row], K1);
    r.left = K1 - K0;
    if (r.left == 0u) return r;
    uint32_t lead;  // bytes from the start of the first piece to the row's first codeword
    if (M.lanes) {
        const int lanes = (int)M.lanes, base = M.rows / lanes, extra = M.rows - base * lanes;
        const int split = extra * (base + 1);  // rows below it belong to lanes that own base + 1 rows
        int g, ra;
        if (row < split) {
            g = row / (base + 1);
            ra = g * (base + 1);
        } else {
            g = extra + (row - split) / max(base, 1);
            ra = split + (g - extra) * base;
        }
        const uint32_t before = K0 - min(row_off[ra], K0);  // the lane's codewords ahead of this row
        r.pp += 16u * ((uintptr_t)((gp_u32)M.wave_off)[g >> 6] + (uintptr_t)(g & 63) + 64u * (uintptr_t)(before >> 3));
        lead = 2u * (before & 7u);
    } else {
        const uintptr_t first_byte = r.pp + 2 * (uintptr_t)K0;
        lead = (uint32_t)(first_byte & 15u);
        r.pp = first_byte - lead;
    }
    r.sub = lead >> 1;
    r.last = r.pp + r.pstride * (uintptr_t)(((lead + 2u * r.left + 15u) >> 4) - 1u);
    return r;
}

// What the two low bits of a device-order code flip in its entry: bit 0 -> bit 18, bit 1 -> bit 26
// (the sign bits of fields 1 and 2).  Written as one shift-or instruction: left to itself the
// compiler turns the two shifts into a 32-bit multiply, which runs at a quarter of the rate.
__device__ __forceinline__ uint32_t order_flips(uint32_t code)
{
    const uint32_t two = code & 3u;
    uint32_t f;
    asm("v_lshl_or_b32 %0, %1, 25, %2" : "=v"(f) : "v"(two), "v"(two << 18));
    return f & ((1u << 18) | (1u << 26));
}

template <typename TablePtr>
__device__ __forceinline__ uint32_t order_entry(TablePtr table, uint32_t code, uint32_t n_groups, uint32_t n_order)
{
    const uint32_t u = max(code >> 2, __builtin_elementwise_sub_sat(code, 3u * n_groups));
    return table[min(u, n_order - 1u)] ^ order_flips(code);
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
// 2 / 4 / 8 tokens: packed, 8 / 8 / 16 bytes per column (a tile of two is staged as a
// tile of four whose last two tokens are not read).
template <int TBI>
__device__ __forceinline__ void lds_load_x(uint32_t xs_addr, uint32_t rec8, float (&v)[TBI])
{
    typedef const __attribute__((address_space(3))) uint32_t *p32;
    if constexpr (TBI == 1) {
        v[0] = __uint_as_float((uint32_t)(*(lp_u16)(uintptr_t)(xs_addr + rec8 + 2u)) << 16);
    } else if constexpr (TBI == 2) {
        const uint32_t u = *(p32)(uintptr_t)(xs_addr + rec8);
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

// The same for a run entry and a tile of 2, 4 or 8 tokens, without widening a value: the
// gathered words hold two tokens' bf16 activations of one column each; a byte permute pairs the
// values that fields 1 and 2 select for one token, and one packed dot product multiplies
// them with the two weights, which are made from the entry's weight bits as bf16 +-2.0 or 0
// (bit 14 = non-zero, bit 15 = negative: 0x4000 / 0xC000): the sums come out doubled, exactly,
// and the caller halves the row scale.  Field 0 takes a dot product with (weight, 0) and
// (0, weight).  Per codeword: three gathers, TBI / 2 * 2 permutes and 2 * TBI dot products.
template <int TBI, int ASYM = 0>
__device__ __forceinline__ void accumulate_tile(uint32_t e0, uint32_t xs_addr, uint32_t pos8,
                                                float (&acc)[TBI * (1 + ASYM)])
{
    static_assert(TBI == 2 || TBI == 4 || TBI == 8, "tile sizes");
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef const __attribute__((address_space(3))) uint32_t *p32;
    constexpr int NW = TBI / 2;             // words per column that are read
    const uint32_t ec = e0 & 0xF8F8F800u;   // byte 1 + z: 8 * position of field z
    const uint32_t t5 = e0 << 5;
    uint32_t w[3];                          // weight pairs: (field 1, field 2), (field 0, 0), (0, field 0)
    w[0] = (t5 & 0xC0000000u) | ((e0 >> 3) & 0x0000C000u);
    w[1] = t5 & 0x0000C000u;
    w[2] = w[1] << 16;
    uint32_t g[3][NW];
#pragma unroll
    for (int z = 0; z < 3; z++) {
        const uint32_t at = pos8 + ((ec >> (8 + 8 * z)) & 0xFFu);
        p32 p = (p32)(uintptr_t)(xs_addr + (TBI == 8 ? 2u * at : at));
#pragma unroll
        for (int k = 0; k < NW; k++) g[z][k] = p[k];
    }
    auto dot = [](uint32_t x2, uint32_t w2, float c) -> float {
        bf16x2 a, b;
        __builtin_memcpy(&a, &x2, 4);
        __builtin_memcpy(&b, &w2, 4);
        return __builtin_amdgcn_fdot2_f32_bf16(a, b, c, false);
    };
#pragma unroll
    for (int k = 0; k < NW; k++) {
        // {g2, g1} as eight bytes: g1 = bytes 0..3, g2 = bytes 4..7
        const uint32_t even = __builtin_amdgcn_perm(g[2][k], g[1][k], 0x05040100u);  // token 2k: (field 1, field 2)
        const uint32_t odd = __builtin_amdgcn_perm(g[2][k], g[1][k], 0x07060302u);   // token 2k + 1
        acc[2 * k] = dot(g[0][k], w[1], dot(even, w[0], acc[2 * k]));
        acc[2 * k + 1] = dot(g[0][k], w[2], dot(odd, w[0], acc[2 * k + 1]));
        if constexpr (ASYM) {
            // the same inputs under |weight|
            const uint32_t m = 0x40004000u;
            acc[TBI + 2 * k] = dot(g[0][k], w[1] & m, dot(even, w[0] & m, acc[TBI + 2 * k]));
            acc[TBI + 2 * k + 1] = dot(g[0][k], w[2] & m, dot(odd, w[0] & m, acc[TBI + 2 * k + 1]));
        }
    }
}

}  // namespace qmoe
