// HIP kernels for gfx950 (CDNA4, wave64) and their launch code.
//
// Work decomposition of the fused decode + product kernel (Section 4.3.3 of the
// paper defines what is computed; the mapping below is this library's own):
//  - a 16-lane DPP row ("group") owns one matrix row at a time; each lane takes
//    one codeword per step, so a step covers 16 consecutive codewords = 32
//    contiguous bytes of the stream, four rows per wavefront;
//  - the running column index of the paper's sequential decoder becomes an
//    inclusive prefix sum of the run lengths inside the group (four DPP row
//    shifts), with the previous step's total carried in through lane 0;
//  - a codeword is looked up in a compact "run entry" table (length plus up to
//    three signed non-zero positions), so the arithmetic per codeword is three
//    gathers from the activations in LDS, not 28 multiply-adds;
//  - the activations of up to eight tokens sit interleaved in LDS as fp32, so
//    one decoded weight is applied to all tokens of the tile with one LDS read;
//  - workgroups are persistent and walk a list of (expert, token tile, row
//    block) items that the dispatch kernel wrote; experts without tokens never
//    appear in it.
#include <hip/hip_runtime.h>

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
constexpr uint32_t kMaxCodes = 0xFFFFFF00u;  // keeps `kb += 16` from wrapping

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

template <int TBI>
__device__ __forceinline__ void lds_load_tile(const float *xs, int col, float (&v)[TBI])
{
    if constexpr (TBI == 1) {
        v[0] = xs[col];
    } else if constexpr (TBI == 2) {
        const float2 t = reinterpret_cast<const float2 *>(xs)[col];
        v[0] = t.x; v[1] = t.y;
    } else if constexpr (TBI == 4) {
        const float4 t = reinterpret_cast<const float4 *>(xs)[col];
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        const float4 t0 = reinterpret_cast<const float4 *>(xs)[2 * col];
        const float4 t1 = reinterpret_cast<const float4 *>(xs)[2 * col + 1];
        v[0] = t0.x; v[1] = t0.y; v[2] = t0.z; v[3] = t0.w;
        v[4] = t1.x; v[5] = t1.y; v[6] = t1.z; v[7] = t1.w;
    }
}

// Decode one step (one codeword per lane) and return this lane's run:
// `len` values starting at column `start` (absolute, clamped to cols).
struct Step {
    uint32_t e0, e1;  // run entry (e0) or interchange words (e0,e1)
    int start, len;
};

template <bool RUN>
__device__ __forceinline__ Step decode_step(const ProductArgs &a, const uint16_t *codes, uint32_t k,
                                            uint32_t kend, int l16, int &incl, const uint32_t *lds_run)
{
    Step s;
    s.e0 = 0; s.e1 = 0;
    if (k < kend) {
        const uint32_t code = codes[k];
        if constexpr (RUN) {
            if (lds_run != nullptr && (int)code < a.lds_dict_entries)
                s.e0 = lds_run[code];
            else
                s.e0 = a.run[code];
        } else {
            const uint2 w = reinterpret_cast<const uint2 *>(a.words)[code];
            s.e0 = w.x; s.e1 = w.y;
        }
    }
    s.len = RUN ? (int)(s.e0 & 31u) : 2 * (int)(s.e0 & 15u);
    // previous step's total sits in lane 15 of the row; lane 0 takes it in
    const int carry = __builtin_amdgcn_update_dpp(0, incl, kRowRor1, 0xf, 0xf, false);
    incl = row_scan16(s.len + (l16 == 0 ? carry : 0));
    s.start = (int)min((uint32_t)(incl - s.len), (uint32_t)a.cols);  // also catches a wrapped index
    return s;
}

template <int TBI, bool RUN>
__device__ __forceinline__ void accumulate_step(const Step &s, const float *xs, float (&acc)[TBI])
{
    if constexpr (RUN) {
#pragma unroll
        for (int j = 0; j < kRunMaxNonzeros; j++) {
            const int sh = kRunLenBits + kRunFieldBits * j;
            const int pos = (int)((s.e0 >> sh) & 31u);
            const int wi = ((int)(s.e0 << (32 - (sh + 7)))) >> 30;  // signed 2-bit weight
            const float w = (float)wi;
            float xv[TBI];
            lds_load_tile<TBI>(xs, s.start + pos, xv);
#pragma unroll
            for (int t = 0; t < TBI; t++) acc[t] = fmaf(w, xv[t], acc[t]);
        }
    } else {
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const uint32_t w = h ? s.e1 : s.e0;
            uint32_t m = ((w >> 4) | (w >> 5)) & 0x05555555u;  // bit 2j set <=> symbol j non-zero
            while (m) {
                const int b = __ffs((int)m) - 1;
                m &= m - 1;
                const int sym = (int)((w >> (4 + b)) & 3u);
                const float wt = sym == 2 ? 1.0f : (sym == 1 ? -1.0f : 0.0f);
                float xv[TBI];
                lds_load_tile<TBI>(xs, s.start + 14 * h + (b >> 1), xv);
#pragma unroll
                for (int t = 0; t < TBI; t++) acc[t] = fmaf(wt, xv[t], acc[t]);
            }
        }
    }
}

template <int TBI, bool RUN, int EPI>
__device__ __forceinline__ void product_rows(const ProductArgs &a, const qmoe_matrix &M, int ntok,
                                             int slot0, int r0, int r1, const float *xs,
                                             const int *tok_ids, const uint32_t *lds_run)
{
    const int l16 = threadIdx.x & 15, grp = threadIdx.x >> 4, ngrp = blockDim.x >> 4;
    for (int r = r0 + grp; r < r1; r += ngrp) {
        const uint32_t kend = min(min(M.row_off[r + 1], M.n_codes), kMaxCodes);
        const uint32_t kbeg = min(M.row_off[r], kend);
        float acc[TBI];
#pragma unroll
        for (int t = 0; t < TBI; t++) acc[t] = 0.0f;
        int incl = 0;
        for (uint32_t kb = kbeg; kb < kend; kb += 16) {
            const Step s = decode_step<RUN>(a, M.codes, kb + l16, kend, l16, incl, lds_run);
            accumulate_step<TBI, RUN>(s, xs, acc);
        }
#pragma unroll
        for (int t = 0; t < TBI; t++) acc[t] = row_sum16_to_last(acc[t]);
        if (l16 == 15) {
            const float scale = half_bits_to_float(M.scale_f16[r]);
#pragma unroll
            for (int t = 0; t < TBI; t++) {
                if (t < ntok) {
                    const float v = acc[t] * scale;
                    if constexpr (EPI == 0) {
                        const int tok = tok_ids[t];
                        const float g = a.gate ? a.gate[tok] : 1.0f;
                        reinterpret_cast<float *>(a.out)[(size_t)tok * a.ld_out + r] = g * v;
                    } else {
                        const float h = v > 0.0f ? v : 0.0f;
                        reinterpret_cast<uint16_t *>(a.out)[(size_t)(slot0 + t) * a.ld_out + r] =
                            float_to_bf16_bits(h);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------- fused decode + product

// EPI 0: fp32 out[token][r] = gate * s_r * acc      (second product, and the plain matvec)
// EPI 1: bf16 out[slot][r]  = relu(s_r * acc)        (first product, writes the hidden vector)
template <bool RUN, int EPI>
__global__ __launch_bounds__(1024) void k_product(const ProductArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float *xs = reinterpret_cast<float *>(smem);
    const size_t xs_bytes = (size_t)(a.cols + kPadCols) * a.tb_max * sizeof(float);
    int *tok_ids = reinterpret_cast<int *>(smem + xs_bytes);            // [kMaxTokenTile] output token
    int *x_rows = tok_ids + kMaxTokenTile;                              // [kMaxTokenTile] input row
    uint32_t *lds_run = a.lds_dict_entries > 0 ? reinterpret_cast<uint32_t *>(smem + xs_bytes + 64) : nullptr;

    int n_pass;
    if (a.items) {
        n_pass = min(*a.n_items_dev, a.max_items);
    } else {
        n_pass = (a.batch + a.tb_max - 1) / a.tb_max;
    }
    const long long total = (long long)n_pass * a.blocks_per_pass;
    const long long per = (total + gridDim.x - 1) / gridDim.x;
    const long long g0 = per * blockIdx.x;
    const long long g1 = min(total, g0 + per);
    if (g0 >= g1) return;

    if (lds_run) {
        for (int i = threadIdx.x; i < a.lds_dict_entries; i += blockDim.x) lds_run[i] = a.run[i];
    }

    int cur_pass = -1, ntok = 0, slot0 = 0, expert = 0, tbi = 1;
    for (long long g = g0; g < g1; g++) {
        const int pass = (int)(g / a.blocks_per_pass);
        const int blk = (int)(g - (long long)pass * a.blocks_per_pass);
        if (pass != cur_pass) {
            __syncthreads();  // everyone is done with the previous tile's activations
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
            }
            __syncthreads();
            for (int c = threadIdx.x; c < a.cols + kPadCols; c += blockDim.x) {
                for (int t = 0; t < tbi; t++) {
                    float v = 0.0f;
                    if (c < a.cols && t < ntok) v = bf16_bits_to_float(a.x[(size_t)x_rows[t] * a.ldx + c]);
                    xs[(size_t)c * tbi + t] = v;
                }
            }
            __syncthreads();
            cur_pass = pass;
        }
        if (ntok == 0) continue;
        const qmoe_matrix M = a.mats ? a.mats[expert] : a.single;
        const int r0 = blk * a.rows_per_item;
        const int r1 = min(a.rows, r0 + a.rows_per_item);
        switch (tbi) {
        case 1: product_rows<1, RUN, EPI>(a, M, ntok, slot0, r0, r1, xs, tok_ids, lds_run); break;
        case 2: product_rows<2, RUN, EPI>(a, M, ntok, slot0, r0, r1, xs, tok_ids, lds_run); break;
        case 4: product_rows<4, RUN, EPI>(a, M, ntok, slot0, r0, r1, xs, tok_ids, lds_run); break;
        default: product_rows<8, RUN, EPI>(a, M, ntok, slot0, r0, r1, xs, tok_ids, lds_run); break;
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
            const Step s = decode_step<RUN>(a, M.codes, kb + l16, kend, l16, incl, nullptr);
            for (int j = 0; j < s.len; j++) {
                int v = 0;
                if constexpr (RUN) {
#pragma unroll
                    for (int z = 0; z < kRunMaxNonzeros; z++) {
                        const int sh = kRunLenBits + kRunFieldBits * z;
                        const int pos = (int)((s.e0 >> sh) & 31u);
                        const int wi = ((int)(s.e0 << (32 - (sh + 7)))) >> 30;
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
    Item *items_wi, *items_wo;
    int tb_wi, tb_wo;
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

// One workgroup of 1024 threads groups the tokens by expert (stable) and writes
// the work lists of both products.
__global__ __launch_bounds__(1024) void k_dispatch(const DispatchArgs a)
{
    extern __shared__ int sm[];
    int *cnt = sm;                 // [E] token count, later the write cursor of each expert
    int *tmp = sm + a.n_experts;   // [32]
    const int E = a.n_experts, T = a.n_tokens;
    const int tid = threadIdx.x, nthr = blockDim.x;

    for (int e = tid; e < E; e += nthr) cnt[e] = 0;
    __syncthreads();
    int dropped = 0;
    for (int t = tid; t < T; t += nthr) {
        const int e = a.expert_idx[t];
        if (e >= 0 && e < E) {
            atomicAdd(&cnt[e], 1);
        } else {
            dropped++;
            if (a.y)
                for (int c = 0; c < a.d_model; c++) a.y[(size_t)t * a.d_model + c] = 0.0f;
        }
    }
    __syncthreads();

    // each thread owns a contiguous chunk of experts
    const int chunk = (E + nthr - 1) / nthr;
    const int e0 = min(E, tid * chunk), e1 = min(E, e0 + chunk);
    int s_tok = 0, s_act = 0, s_wi = 0, s_wo = 0;
    for (int e = e0; e < e1; e++) {
        const int n = cnt[e];
        s_tok += n;
        s_act += n > 0;
        s_wi += (n + a.tb_wi - 1) / a.tb_wi;
        s_wo += (n + a.tb_wo - 1) / a.tb_wo;
    }
    int tot_tok, tot_act, tot_wi, tot_wo, tot_drop;
    int p_tok = block_exclusive_scan(s_tok, tmp, tot_tok);
    block_exclusive_scan(s_act, tmp, tot_act);
    int p_wi = block_exclusive_scan(s_wi, tmp, tot_wi);
    int p_wo = block_exclusive_scan(s_wo, tmp, tot_wo);
    block_exclusive_scan(dropped, tmp, tot_drop);
    for (int e = e0; e < e1; e++) {
        const int n = cnt[e];
        a.tok_off[e] = p_tok;
        for (int i = 0; i * a.tb_wi < n; i++)
            a.items_wi[p_wi++] = Item{e, p_tok + i * a.tb_wi, min(a.tb_wi, n - i * a.tb_wi), 0};
        for (int i = 0; i * a.tb_wo < n; i++)
            a.items_wo[p_wo++] = Item{e, p_tok + i * a.tb_wo, min(a.tb_wo, n - i * a.tb_wo), 0};
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
        a.counters[5] = 0; a.counters[6] = 0; a.counters[7] = 0;
    }
    __syncthreads();

    // Stable scatter.  A wavefront takes 64 consecutive tokens; inside it a token's
    // rank among equal experts is counted by broadcasting every lane once.  The
    // wavefronts then append their tokens one after the other, in token order.
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthr >> 6;
    for (int base = 0; base < T; base += nthr) {
        const int t = base + tid;
        int e = -1;
        if (t < T) {
            e = a.expert_idx[t];
            if (e < 0 || e >= E) e = -1;
        }
        int rank = 0, same = 0;
        for (int j = 0; j < 64; j++) {
            const int ej = __shfl(e, j, 64);
            const int m = (ej == e) ? 1 : 0;
            same += m;
            rank += (j < lane) ? m : 0;
        }
        for (int w = 0; w < nwaves; w++) {
            if (w == wave && e >= 0) {
                const int cur = cnt[e];
                a.perm[cur + rank] = t;
                if (rank == same - 1) cnt[e] = cur + same;
            }
            __syncthreads();
        }
    }
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
};

template <int TBI>
__device__ __forceinline__ void dense_rows(const DenseArgs &a, const uint16_t *W, int ntok, int slot0,
                                           int r0, int r1, const float *xs, const int *tok_ids)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    for (int r = r0 + wave; r < r1; r += nwaves) {
        const uint4 *wrow = reinterpret_cast<const uint4 *>(W + (size_t)r * a.cols);
        float acc[TBI];
#pragma unroll
        for (int t = 0; t < TBI; t++) acc[t] = 0.0f;
        for (int c8 = lane; c8 < a.cols / 8; c8 += 64) {
            const uint4 q = wrow[c8];
            const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const float w0 = __uint_as_float(u[i] << 16), w1 = __uint_as_float(u[i] & 0xFFFF0000u);
                float x0[TBI], x1[TBI];
                lds_load_tile<TBI>(xs, c8 * 8 + 2 * i, x0);
                lds_load_tile<TBI>(xs, c8 * 8 + 2 * i + 1, x1);
#pragma unroll
                for (int t = 0; t < TBI; t++) acc[t] = fmaf(w1, x1[t], fmaf(w0, x0[t], acc[t]));
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
    const size_t xs_bytes = (size_t)(a.cols + kPadCols) * a.tb_max * sizeof(float);
    int *tok_ids = reinterpret_cast<int *>(smem + xs_bytes);
    int *x_rows = tok_ids + kMaxTokenTile;

    const int n_pass = min(*a.n_items_dev, a.max_items);
    const long long total = (long long)n_pass * a.blocks_per_pass;
    const long long per = (total + gridDim.x - 1) / gridDim.x;
    const long long g0 = per * blockIdx.x;
    const long long g1 = min(total, g0 + per);
    int cur_pass = -1, ntok = 0, slot0 = 0, expert = 0, tbi = 1;
    for (long long g = g0; g < g1; g++) {
        const int pass = (int)(g / a.blocks_per_pass);
        const int blk = (int)(g - (long long)pass * a.blocks_per_pass);
        if (pass != cur_pass) {
            __syncthreads();
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
            for (int c = threadIdx.x; c < a.cols + kPadCols; c += blockDim.x)
                for (int t = 0; t < tbi; t++) {
                    float v = 0.0f;
                    if (c < a.cols && t < ntok) v = bf16_bits_to_float(a.x[(size_t)x_rows[t] * a.ldx + c]);
                    xs[(size_t)c * tbi + t] = v;
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
        case 1: dense_rows<1>(a, W, ntok, slot0, r0, r1, xs, tok_ids); break;
        case 2: dense_rows<2>(a, W, ntok, slot0, r0, r1, xs, tok_ids); break;
        case 4: dense_rows<4>(a, W, ntok, slot0, r0, r1, xs, tok_ids); break;
        default: dense_rows<8>(a, W, ntok, slot0, r0, r1, xs, tok_ids); break;
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

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct ProductPlan {
    int threads, rows_per_item, blocks_per_pass, tb_max, lds_dict_entries, grid;
    size_t smem;
};

// Pick the token tile, workgroup size and grid for a product over rows x cols matrices.
qmoe_status plan_product(int rows, int cols, bool run_table, long long max_passes_hint, ProductPlan *p)
{
    DeviceInfo di;
    const qmoe_status st = device_info(&di);
    if (st != QMOE_OK) return st;
    const Tuning &tu = tuning();
    const size_t col_bytes = (size_t)(cols + kPadCols) * sizeof(float);
    // activations of one tile should leave room for a second workgroup on the CU
    size_t budget = (size_t)di.max_lds / 2 - 256;
    int tb = kMaxTokenTile;
    while (tb > 1 && col_bytes * tb > budget) tb >>= 1;
    if (tu.token_tile > 0) {
        tb = 1;
        while (tb * 2 <= tu.token_tile && tb < kMaxTokenTile) tb <<= 1;
    }
    if (col_bytes * tb + 256 > (size_t)di.max_lds) return QMOE_E_LIMIT;
    int lds_dict = 0;
    if (run_table && tu.lds_dict_entries > 0) {
        lds_dict = std::min(tu.lds_dict_entries, kTableEntries);
        while (tb > 1 && col_bytes * tb + 64 + 4 * (size_t)lds_dict > (size_t)di.max_lds) tb >>= 1;
        if (col_bytes * tb + 64 + 4 * (size_t)lds_dict > (size_t)di.max_lds)
            lds_dict = (int)(((size_t)di.max_lds - col_bytes * tb - 64) / 4);
    }
    p->tb_max = tb;
    p->lds_dict_entries = lds_dict;
    p->smem = col_bytes * tb + 64 + 4 * (size_t)lds_dict;
    int threads = tu.threads > 0 ? tu.threads : (p->smem * 2 > (size_t)di.max_lds ? 1024 : 512);
    threads = std::max(64, std::min(1024, threads / 64 * 64));
    p->threads = threads;
    int rpi = tu.rows_per_item > 0 ? tu.rows_per_item : 4 * (threads / 16);
    rpi = std::max(1, std::min(rpi, rows));
    p->rows_per_item = rpi;
    p->blocks_per_pass = (rows + rpi - 1) / rpi;
    const int wg_per_cu = tu.grid_per_cu > 0 ? tu.grid_per_cu
                                             : std::max(1, std::min((int)((size_t)di.max_lds / p->smem), 2048 / threads));
    long long grid = (long long)di.cus * wg_per_cu;
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

template <bool RUN, int EPI>
qmoe_status launch_product_as(const ProductArgs &a, const ProductPlan &p, hipStream_t s)
{
    const qmoe_status st = allow_lds(k_product<RUN, EPI>, p.smem);
    if (st != QMOE_OK) return st;
    hipLaunchKernelGGL((k_product<RUN, EPI>), dim3(p.grid), dim3(p.threads), p.smem, s, a);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

qmoe_status launch_product(const ProductArgs &a, const ProductPlan &p, bool run, hipStream_t s)
{
    if (run) return a.epilogue ? launch_product_as<true, 1>(a, p, s) : launch_product_as<true, 0>(a, p, s);
    return a.epilogue ? launch_product_as<false, 1>(a, p, s) : launch_product_as<false, 0>(a, p, s);
}

qmoe_status check_matrix_args(const qmoe_dict *d, const qmoe_matrix *W)
{
    if (!d || !W) return QMOE_E_INVALID_ARG;
    if (!W->codes || !W->row_off || !W->scale_f16 || W->rows < 1 || W->cols < 2 || (W->cols & 1))
        return QMOE_E_INVALID_ARG;
    if (W->cols > kMaxCols) return QMOE_E_LIMIT;
    if (!d->dev) return QMOE_E_NO_DEVICE_DICT;
    return QMOE_OK;
}

void fill_tables(const qmoe_dict *d, ProductArgs *a)
{
    const unsigned char *base = static_cast<const unsigned char *>(d->dev);
    a->run = reinterpret_cast<const uint32_t *>(base + kDevRunOffset);
    a->words = reinterpret_cast<const uint32_t *>(base + kDevWordsOffset);
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
    Item *items_wi, *items_wo;
    uint16_t *hidden;
};

LayerPtrs layer_ptrs(void *ws, const qmoe_ws_layout &l)
{
    unsigned char *b = static_cast<unsigned char *>(ws);
    return LayerPtrs{reinterpret_cast<int *>(b + l.tok_off), reinterpret_cast<int *>(b + l.perm),
                     reinterpret_cast<int *>(b + l.counters), reinterpret_cast<Item *>(b + l.items_wi),
                     reinterpret_cast<Item *>(b + l.items_wo), reinterpret_cast<uint16_t *>(b + l.hidden)};
}

qmoe_status launch_dispatch(const int32_t *expert_idx, int n_tokens, int n_experts, int d_model,
                            const LayerPtrs &lp, int tb_wi, int tb_wo, float *y, hipStream_t s)
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
    da.tb_wi = tb_wi;
    da.tb_wo = tb_wo;
    da.y = y;
    da.d_model = d_model;
    const size_t smem = sizeof(int) * ((size_t)n_experts + 32);
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
    d->dev = dev_buf;
    return QMOE_OK;
}

qmoe_status qmoe_decode_matvec(const qmoe_dict *d, const qmoe_matrix *W, const uint16_t *x_bf16, int batch,
                               float *y, void *stream)
{
    qmoe_status st = check_matrix_args(d, W);
    if (st != QMOE_OK) return st;
    if (!x_bf16 || !y || batch < 1) return QMOE_E_INVALID_ARG;
    const bool run = d->max_nonzeros <= kRunMaxNonzeros;
    ProductPlan p;
    if ((st = plan_product(W->rows, W->cols, run, ((long long)batch + 7) / 8 + 1, &p)) != QMOE_OK) return st;
    // grid sized for the real number of tiles
    {
        const long long items = (long long)((batch + p.tb_max - 1) / p.tb_max) * p.blocks_per_pass;
        if (items < p.grid) p.grid = (int)std::max(1LL, items);
    }
    ProductArgs a{};
    a.mats = nullptr;
    a.single = *W;
    fill_tables(d, &a);
    a.items = nullptr;
    a.n_items_dev = nullptr;
    a.max_items = 0;
    a.n_experts = 1;
    a.batch = batch;
    a.perm = nullptr;
    a.x = x_bf16;
    a.x_by_slot = 1;
    a.ldx = W->cols;
    a.out = y;
    a.ld_out = W->rows;
    a.gate = nullptr;
    a.epilogue = 0;
    a.rows = W->rows;
    a.cols = W->cols;
    a.rows_per_item = p.rows_per_item;
    a.blocks_per_pass = p.blocks_per_pass;
    a.tb_max = p.tb_max;
    a.lds_dict_entries = p.lds_dict_entries;
    return launch_product(a, p, run, static_cast<hipStream_t>(stream));
}

qmoe_status qmoe_decode_dense(const qmoe_dict *d, const qmoe_matrix *W, int8_t *out, int path, void *stream)
{
    qmoe_status st = check_matrix_args(d, W);
    if (st != QMOE_OK) return st;
    if (!out || (path != 0 && path != 1)) return QMOE_E_INVALID_ARG;
    const bool run = path == 0 && d->max_nonzeros <= kRunMaxNonzeros;
    ProductArgs a{};
    a.single = *W;
    fill_tables(d, &a);
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

qmoe_status qmoe_moe_layer_ws_layout(int n_experts, int d_model, int d_ff, int n_tokens, qmoe_ws_layout *out)
{
    if (!out) return QMOE_E_INVALID_ARG;
    const qmoe_status st = layer_limits(n_experts, d_model, d_ff, n_tokens);
    if (st != QMOE_OK) return st;
    size_t off = 0;
    out->tok_off = off;  off = align_up(off + sizeof(int) * ((size_t)n_experts + 1), 256);
    out->perm = off;     off = align_up(off + sizeof(int) * (size_t)n_tokens, 256);
    out->counters = off; off = align_up(off + sizeof(int) * 8, 256);
    out->items_wi = off; off = align_up(off + sizeof(Item) * (size_t)n_tokens, 256);
    out->items_wo = off; off = align_up(off + sizeof(Item) * (size_t)n_tokens, 256);
    out->hidden = off;   off = align_up(off + sizeof(uint16_t) * (size_t)n_tokens * (size_t)d_ff, 256);
    out->total = off;
    return QMOE_OK;
}

size_t qmoe_moe_layer_workspace(int n_experts, int d_model, int d_ff, int n_tokens)
{
    qmoe_ws_layout l;
    return qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens, &l) == QMOE_OK ? l.total : 0;
}

qmoe_status qmoe_moe_dispatch(const int32_t *expert_idx, int n_tokens, int n_experts, int d_model, int d_ff,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    qmoe_ws_layout l;
    qmoe_status st = qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens, &l);
    if (st != QMOE_OK) return st;
    if (!expert_idx) return QMOE_E_INVALID_ARG;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < l.total)
        return QMOE_E_WORKSPACE;
    ProductPlan pwi, pwo;
    if ((st = plan_product(d_ff, d_model, true, n_tokens, &pwi)) != QMOE_OK) return st;
    if ((st = plan_product(d_model, d_ff, true, n_tokens, &pwo)) != QMOE_OK) return st;
    return launch_dispatch(expert_idx, n_tokens, n_experts, d_model, layer_ptrs(workspace, l), pwi.tb_max,
                           pwo.tb_max, nullptr, static_cast<hipStream_t>(stream));
}

qmoe_status qmoe_moe_layer_forward(const qmoe_dict *d, const qmoe_matrix *wi, const qmoe_matrix *wo,
                                   int n_experts, int d_model, int d_ff, const uint16_t *x_bf16,
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
    const bool run = d->max_nonzeros <= kRunMaxNonzeros;
    ProductPlan pwi, pwo;
    if ((st = plan_product(d_ff, d_model, run, n_tokens, &pwi)) != QMOE_OK) return st;
    if ((st = plan_product(d_model, d_ff, run, n_tokens, &pwo)) != QMOE_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const LayerPtrs lp = layer_ptrs(workspace, l);
    const int phases = tuning().phases > 0 ? tuning().phases : 7;
    if (phases & 1)
        if ((st = launch_dispatch(expert_idx, n_tokens, n_experts, d_model, lp, pwi.tb_max, pwo.tb_max, y, s)) !=
            QMOE_OK)
            return st;

    ProductArgs a{};
    fill_tables(d, &a);
    a.n_experts = n_experts;
    a.max_items = n_tokens;
    a.perm = lp.perm;
    a.gate = nullptr;
    // first product: hidden[slot] = bf16(relu(Wi x[token]))
    a.mats = wi;
    a.items = lp.items_wi;
    a.n_items_dev = lp.counters + 3;
    a.x = x_bf16;
    a.x_by_slot = 0;
    a.ldx = d_model;
    a.out = lp.hidden;
    a.ld_out = d_ff;
    a.epilogue = 1;
    a.rows = d_ff;
    a.cols = d_model;
    a.rows_per_item = pwi.rows_per_item;
    a.blocks_per_pass = pwi.blocks_per_pass;
    a.tb_max = pwi.tb_max;
    a.lds_dict_entries = pwi.lds_dict_entries;
    if (phases & 2)
        if ((st = launch_product(a, pwi, run, s)) != QMOE_OK) return st;
    // second product: y[token] = gate * Wo hidden[slot]
    a.mats = wo;
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
    a.lds_dict_entries = pwo.lds_dict_entries;
    if (phases & 4) return launch_product(a, pwo, run, s);
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
    if ((st = plan_product(d_ff, d_model, false, n_tokens, &pwi)) != QMOE_OK) return st;
    if ((st = plan_product(d_model, d_ff, false, n_tokens, &pwo)) != QMOE_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const LayerPtrs lp = layer_ptrs(workspace, l);
    const int phases = tuning().phases > 0 ? tuning().phases : 7;
    if (phases & 1)
        if ((st = launch_dispatch(expert_idx, n_tokens, n_experts, d_model, lp, pwi.tb_max, pwo.tb_max, y, s)) !=
            QMOE_OK)
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
    if (phases & 4) {
        if ((st = allow_lds(k_dense_bf16, pwo.smem)) != QMOE_OK) return st;
        hipLaunchKernelGGL(k_dense_bf16, dim3(pwo.grid), dim3(pwo.threads), pwo.smem, s, a);
        QMOE_HIP_TRY(hipGetLastError());
    }
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
