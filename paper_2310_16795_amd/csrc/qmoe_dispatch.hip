// Step one of a layer call: tokens grouped by expert (stable), experts without tokens
// skipped (Section 5.1 of the paper), work lists for the product kernels.
#include "qmoe_dev.h"

namespace qmoe {
namespace {

// ---------------------------------------------------------------- dispatch


// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel-primitive adds (no trip
// through the LDS crossbar): the row scan, then lane 15 of a row added to the whole next row, then
// lane 31 to the upper half.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp_add(int x)
{
    return x + __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xf, false);  // lanes without a source add 0
}
__device__ __forceinline__ int wave_inclusive_scan(int x)
{
    x = row_scan16(x);
    x = dpp_add<0x142, 0xa>(x);  // row_bcast:15 into rows 1 and 3
    x = dpp_add<0x143, 0xc>(x);  // row_bcast:31 into rows 2 and 3
    return x;
}

// Exclusive prefix sums of N ints per thread over the workgroup (up to 16 wavefronts), all at
// once (three barriers).  `tmp` holds >= 17 * N ints: [value][wavefront], then the N totals.
template <int N>
__device__ __forceinline__ void block_exclusive_scan_n(const int (&v)[N], int *tmp, int (&excl)[N], int (&total)[N])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = (blockDim.x + 63) >> 6;
    int incl[N];
#pragma unroll
    for (int k = 0; k < N; k++) {
        incl[k] = wave_inclusive_scan(v[k]);
        if (lane == 63) tmp[k * 16 + wave] = incl[k];
    }
    __syncthreads();
    if (wave == 0) {
        // a row of 16 lanes per value: lane w of the row holds wavefront w's sum; four values a turn
        for (int k0 = 0; k0 < N; k0 += 4) {
            const int k = k0 + (lane >> 4), w = lane & 15;
            const bool live = k < N && w < nwaves;
            const int mine = live ? tmp[k * 16 + w] : 0;
            const int run = row_scan16(mine);
            if (live) tmp[k * 16 + w] = run - mine;
            if (k < N && w == 15) tmp[16 * N + k] = run;  // wavefronts that do not exist added 0
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < N; k++) {
        excl[k] = tmp[k * 16 + wave] + incl[k] - v[k];
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

}  // namespace

qmoe_status launch_dispatch_kernel(const DispatchArgs &da, hipStream_t s)
{
    // token counts, scan scratch (17 x 12, rounded up), two arrays of one round of tokens
    const size_t smem = sizeof(int) * ((size_t)da.n_experts + 256 + 2 * 1024);
    const qmoe_status st = allow_lds(k_dispatch, smem);
    if (st != QMOE_OK) return st;
    // small layers: fewer wavefronts meet at the kernel's barriers and the scan has fewer partial sums
    const int need = da.n_tokens > da.n_experts ? da.n_tokens : da.n_experts;
    const int threads = need <= 256 ? 256 : (need <= 512 ? 512 : 1024);
    hipLaunchKernelGGL(k_dispatch, dim3(1), dim3(threads), smem, s, da);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

}  // namespace qmoe
