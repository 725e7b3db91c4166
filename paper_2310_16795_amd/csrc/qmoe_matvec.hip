// One matrix at a time: the latency-oriented product of qmoe_decode_matvec (16 lanes per
// matrix row) and the decode-only hook that shows the stream is read bit-exactly.
#include "qmoe_dev.h"

namespace qmoe {
namespace {

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
            case 2: stage_x_tile<4>(xs_w, a.x, row_of, ntok, a.ldx, a.cols); break;  // eight bytes per column as well
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
        if (kbeg >= kend) {
            // a row without codewords (only a corrupt stream has one) decodes to zeros
            if (l16 == 15)
                for (int t = 0; t < ntok; t++) reinterpret_cast<float *>(a.out)[(size_t)(slot0 + t) * a.ld_out + r] = 0.0f;
            continue;
        }
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
            // A row's steps are a chain (the running column), but what a step needs from memory is not:
            // the codewords are fetched two steps ahead and their table entries one step ahead, from
            // addresses that always exist (a lane past the row's end reads the row's last codeword and
            // drops it), so that only the first step of a row waits for its trips to memory in full.
            int incl = 0;
            gp_u16 codes = (gp_u16)M.codes;
            auto code_at = [&](uint32_t k) -> uint32_t { return (uint32_t)codes[min(k, kend - 1u)]; };
            auto entry_of = [&](uint32_t code) -> Entry {
                Entry e{0u, 0u};
                if constexpr (RUN) {
                    e.e0 = a.code_order ? order_entry((gp_u32)a.order_table, code, (uint32_t)a.n_groups, (uint32_t)a.n_order)
                                        : ((gp_u32)a.run)[code];
                } else {
                    const unsigned long long w = ((gp_u64)a.words)[code];
                    e.e0 = (uint32_t)w; e.e1 = (uint32_t)(w >> 32);
                }
                return e;
            };
            uint32_t c_next = code_at(kbeg + 16u + (uint32_t)l16);
            Entry e_cur = entry_of(code_at(kbeg + (uint32_t)l16));
            for (uint32_t kb = kbeg; kb < kend; kb += 16) {
                const uint32_t c_after = code_at(kb + 32u + (uint32_t)l16);
                const Entry e_next = entry_of(c_next);
                Entry e = e_cur;
                if (kb + (uint32_t)l16 >= kend) { e.e0 = 0u; e.e1 = 0u; }  // past the row's end: an empty run
                const int len = RUN ? (int)((e.e0 & 0xFFu) >> 3) : 2 * (int)(e.e0 & 15u);
                // previous step's total sits in lane 15 of the row; lane 0 takes it in
                const int carry = __builtin_amdgcn_update_dpp(0, incl, kRowRor1, 0xf, 0xf, false);
                incl = row_scan16(len + (l16 == 0 ? carry : 0));
                const uint32_t start = min((uint32_t)(incl - len), (uint32_t)a.cols);  // also catches a wrapped index
                accumulate<TBI, DICT, ASYM>(e, xs_addr, 8u * start, acc);
                e_cur = e_next;
                c_next = c_after;
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

}  // namespace

qmoe_status launch_matvec_rows(const ProductArgs &a, bool run, bool minmax, int grid, int threads, size_t smem,
                               hipStream_t s)
{
    auto launch = [&](auto kernel) -> qmoe_status {
        const qmoe_status lst = allow_lds(kernel, smem);
        if (lst != QMOE_OK) return lst;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), smem, s, a);
        return QMOE_OK;
    };
    qmoe_status st;
    if (minmax)
        st = run ? launch(k_matvec_rows<true, 1>) : launch(k_matvec_rows<false, 1>);
    else
        st = run ? launch(k_matvec_rows<true, 0>) : launch(k_matvec_rows<false, 0>);
    if (st != QMOE_OK) return st;
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

qmoe_status launch_decode_dense(const ProductArgs &a, bool run, int8_t *out, int grid, hipStream_t s)
{
    if (run)
        hipLaunchKernelGGL(k_decode_dense<true>, dim3(grid), dim3(256), 0, s, a, out);
    else
        hipLaunchKernelGGL(k_decode_dense<false>, dim3(grid), dim3(256), 0, s, a, out);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

}  // namespace qmoe
