// Kernels around the hot path: the encoder on the device, the uncompressed bf16
// comparator, a plain copy (bandwidth yardstick) and the load-time renumbering of a stream.
#include "qmoe_dev.h"

namespace qmoe {
namespace {

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

// ---------------------------------------------------------------- encoder
//
// Longest-prefix coding of ternary rows with the dictionary's trie (Section 4.3.3
// "Encoding"), one row per lane: walk pairs from the root while a child exists, emit the
// codeword of the deepest node that ends an entry, continue after that entry.  Three
// launches: count codewords per row, turn the counts into row offsets (one workgroup), write
// the codewords.  Same stream as qmoe_encode_host, codeword for codeword.


__global__ void k_encode_clear(int *status)
{
    if (threadIdx.x < 2) status[threadIdx.x] = 0;
}

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


// One wavefront per row; a lane takes eight consecutive columns at a time (16 bytes of
// weights, 1 KiB per wavefront and load; rows whose width is no multiple of 8: four columns,
// 8 bytes) and the matching activations from token-major fp32 planes in LDS (consecutive
// lanes read consecutive 16-byte pieces).  The weight pointer comes out of an array in memory,
// so it is given its address space by hand: through a generic pointer every load would also
// count as LDS traffic and be waited for together with the reads of the activations.
template <int TBI>
__device__ __forceinline__ void dense_rows(const DenseArgs &a, const uint16_t *W, int ntok, int slot0,
                                           int r0, int r1, const float *xs, int plane, const int *tok_ids)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const uintptr_t wbase = reinterpret_cast<uintptr_t>(W);
    auto fma4 = [&](uint32_t qx, uint32_t qy, int c4, float (&acc)[TBI]) {
        const float w0 = __uint_as_float(qx << 16), w1 = __uint_as_float(qx & 0xFFFF0000u);
        const float w2 = __uint_as_float(qy << 16), w3 = __uint_as_float(qy & 0xFFFF0000u);
#pragma unroll
        for (int t = 0; t < TBI; t++) {
            const float4 x = reinterpret_cast<const float4 *>(xs + (size_t)t * plane)[c4];
            acc[t] = fmaf(w3, x.w, fmaf(w2, x.z, fmaf(w1, x.y, fmaf(w0, x.x, acc[t]))));
        }
    };
    for (int r = r0 + wave; r < r1; r += nwaves) {
        const uintptr_t wrow = wbase + 2 * (size_t)r * a.cols;
        float acc[TBI];
#pragma unroll
        for (int t = 0; t < TBI; t++) acc[t] = 0.0f;
        if ((a.cols & 7) == 0) {
            const int n8 = a.cols / 8;
#pragma unroll 4
            for (int c8 = lane; c8 < n8; c8 += 64) {
                const u32x4 q = ((gp_u32x4)wrow)[c8];
                fma4(q.x, q.y, 2 * c8, acc);
                fma4(q.z, q.w, 2 * c8 + 1, acc);
            }
        } else {
            const int nq = a.cols / 4;
#pragma unroll 4
            for (int c4 = lane; c4 < nq; c4 += 64) {
                const unsigned long long q = ((gp_u64)wrow)[c4];
                fma4((uint32_t)q, (uint32_t)(q >> 32), c4, acc);
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

}  // namespace

qmoe_status launch_encode(const EncodeArgs &a, hipStream_t s)
{
    const int grid = (a.rows + 255) / 256;
    // the status words are cleared by a kernel, not a memset node, so the call can be captured into a HIP graph
    hipLaunchKernelGGL(k_encode_clear, dim3(1), dim3(64), 0, s, a.status);
    hipLaunchKernelGGL(k_encode<false>, dim3(grid), dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_encode_offsets, dim3(1), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(k_encode<true>, dim3(grid), dim3(256), 0, s, a);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

qmoe_status launch_dense_bf16(const DenseArgs &a, const ProductPlan &p, hipStream_t s)
{
    const qmoe_status st = allow_lds(k_dense_bf16, p.smem);
    if (st != QMOE_OK) return st;
    hipLaunchKernelGGL(k_dense_bf16, dim3(p.grid), dim3(p.threads), p.smem, s, a);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

qmoe_status launch_stream_copy(void *dst, const void *src, size_t n16, int grid, hipStream_t s)
{
    hipLaunchKernelGGL(k_stream_copy, dim3(grid), dim3(256), 0, s, static_cast<const uint4 *>(src),
                       static_cast<uint4 *>(dst), n16);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

qmoe_status launch_renumber(uint16_t *codes, size_t n, const uint16_t *map, int grid, hipStream_t s)
{
    hipLaunchKernelGGL(k_renumber, dim3(grid), dim3(256), 0, s, codes, n, map);
    QMOE_HIP_TRY(hipGetLastError());
    return QMOE_OK;
}

}  // namespace qmoe
