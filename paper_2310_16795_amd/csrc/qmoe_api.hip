// Launch planning and the C ABI of the device side (include/qmoe.h).
#include <mutex>

#include "qmoe_dev.h"

namespace qmoe {

std::atomic<int> g_last_hip_error{0};

qmoe_status allow_lds_bytes(const void *kernel, size_t smem)
{
    if (smem > 48 * 1024)
        QMOE_HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    return QMOE_OK;
}

qmoe_status launch_product(const ProductArgs &a, const ProductPlan &p, bool run, hipStream_t s)
{
    return a.minmax ? launch_product_asym(a, p, run, s) : launch_product_sym(a, p, run, s);
}

namespace {



qmoe_status device_info(DeviceInfo *out)
{
    static DeviceInfo cached[64];
    static std::mutex mu;
    int dev = 0;
    QMOE_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return QMOE_E_LIMIT;
    std::lock_guard<std::mutex> lock(mu);
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

// The scalar kernels of a layer run on a second stream, next to the matrix-core kernels.
// The caller may bring that stream; otherwise the library makes one per device on first use
// (default priority) and keeps it until the process ends.  The two events that fork and join
// it are the library's in both cases (one pair per device, made on first use).
struct SideStream {
    hipStream_t stream = nullptr;   // library-owned, made only when a call brings none
    hipEvent_t fork = nullptr, join = nullptr;
    bool events = false;
};

qmoe_status side_stream(hipStream_t callers, SideStream *out)
{
    static SideStream cached[64];
    static std::mutex mu;
    int dev = 0;
    QMOE_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return QMOE_E_LIMIT;
    std::lock_guard<std::mutex> lock(mu);
    SideStream &c = cached[dev];
    if (!c.events) {
        QMOE_HIP_TRY(hipEventCreateWithFlags(&c.fork, hipEventDisableTiming));
        QMOE_HIP_TRY(hipEventCreateWithFlags(&c.join, hipEventDisableTiming));
        c.events = true;
    }
    if (!callers && !c.stream) QMOE_HIP_TRY(hipStreamCreateWithFlags(&c.stream, hipStreamNonBlocking));
    *out = c;
    if (callers) out->stream = callers;
    return QMOE_OK;
}

// Scratch memory of qmoe_moe_layer_forward_static: a bounded workspace that lives in the
// library's own device image, so that the call allocates nothing.  Each GPU holds its own
// copy at its own address; host code uses the address hipGetSymbolAddress returns for the
// current device, never the array's name.
constexpr size_t kStaticWsBytes = (size_t)8 << 20;
__device__ __align__(256) unsigned char g_static_ws[kStaticWsBytes];

qmoe_status static_workspace(void **out)
{
    static void *cached[64];
    static std::mutex mu;
    int dev = 0;
    QMOE_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return QMOE_E_LIMIT;
    std::lock_guard<std::mutex> lock(mu);
    if (!cached[dev]) {
        void *p = nullptr;
        QMOE_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_ws)));
        if (!p) return QMOE_E_HIP;
        cached[dev] = p;
    }
    *out = cached[dev];
    return QMOE_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }


// Pick the token tile, workgroup size, blocks per matrix and grid for a product over rows x cols
// matrices with the lane-per-row kernel (compressed path).
qmoe_status plan_product(int rows, int cols, bool run_table, long long max_passes_hint, ProductPlan *p,
                         int n_order = 0, int force_blocks = 0, int stage_out_row_bytes = 0, bool minmax = false,
                         int force_lanes = 0)
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
    if (force_lanes > 0) {
        // streams in the lane-interleaved layout: workgroups x lanes must be the count the layout was
        // built for; as few workgroups per matrix as the workgroup size allows
        // (the split the search above found if it has that many lanes, else the nearest one that does)
        auto fits = [&](int b) {
            return b >= 1 && force_lanes % b == 0 && (force_lanes / b) % 64 == 0 && force_lanes / b <= max_threads;
        };
        const int want_b = best_b;
        best_b = 0;
        for (int d = 0; d <= force_lanes / 64 && !best_b; d++) {
            if (fits(want_b + d)) best_b = want_b + d;
            else if (fits(want_b - d)) best_b = want_b - d;
        }
        if (!best_b) return QMOE_E_INVALID_ARG;
        best_t = force_lanes / best_b;
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
    // A tile is walked column step by column step by one wavefront per 64 rows: a long chain
    // that pays only when the scalar kernel would need several rounds of items per compute
    // unit anyway.  With few tokens in the call (measured: 512 tokens on 128 experts) the
    // scalar kernel finishes every expert in one round and the chain would be the critical path.
    if (tu.mfma_min_tokens == 0 && n_tokens < 4 * di.cus) return QMOE_OK;
    mp->min_tokens = tu.mfma_min_tokens > 0 ? tu.mfma_min_tokens : kMmMinTokensDefault;
    mp->grid = di.cus;
    mp->smem = mm_lds_bytes(n_order);
    return QMOE_OK;
}

qmoe_status check_matrix_args(const qmoe_dict *d, const qmoe_matrix *W)
{
    if (!d || !W) return QMOE_E_INVALID_ARG;
    if (W->lanes || W->wave_off) return QMOE_E_INVALID_ARG;  // the single-matrix calls read rows back to back
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

// Splits a format argument (QMOE_FORMAT_* bits) into the numbering, the grid and the lane counts
// of the lane-interleaved layout (0, 0 = rows back to back).
qmoe_status split_format(int format, int *code_order, bool *minmax, int *lanes_wi = nullptr, int *lanes_wo = nullptr)
{
    if (format < 0 || (format & ~(QMOE_FORMAT_DEVICE_ORDER | QMOE_FORMAT_GRID_MINMAX | 0xFFFF00))) return QMOE_E_INVALID_ARG;
    *code_order = (format & QMOE_FORMAT_DEVICE_ORDER) ? 1 : 0;
    *minmax = (format & QMOE_FORMAT_GRID_MINMAX) != 0;
    const int lwi = 64 * ((format >> 8) & 0xFF), lwo = 64 * ((format >> 16) & 0xFF);
    if ((lwi || lwo) && (!*code_order || !lwi || !lwo)) return QMOE_E_INVALID_ARG;  // both or neither; device numbering only
    if (lanes_wi) *lanes_wi = lwi;
    if (lanes_wo) *lanes_wo = lwo;
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
    return launch_dispatch_kernel(da, s);
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
    return launch_encode(a, static_cast<hipStream_t>(stream));
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
    // per 8.  Its unit of work is 64 rows of a token tile, taken by one wavefront (a unit's time is
    // set by the length of a row, not by how many units there are).
    {
        const Tuning &tu = tuning();
        const int n_order = (int)d->order_table.size();
        if (code_order == 1 && run && n_order > 0 && tu.mfma_min_tokens >= 0 && W->cols % 8 == 0 &&
            reinterpret_cast<uintptr_t>(x_bf16) % 16 == 0 && mm_lds_bytes(n_order) <= (size_t)di.max_lds) {
            const int tiles = (batch + kMmTokens - 1) / kMmTokens;
            const int waves = kMmThreads / 64;
            const long long units = (long long)tiles * ((W->rows + 63) / 64);
            const long long blocks = (units + waves - 1) / waves;  // workgroups with every wavefront busy
            // Measured on this GPU (microseconds): a round of the matrix-core kernel (every wavefront of
            // every compute unit with one unit of 64 tokens) takes about 8 + 0.0148 per column; the other
            // kernel works through tiles of eight tokens at 1.3 million weights per microsecond with one
            // workgroup resident per compute unit (long rows: the tile's activations fill the LDS) and
            // about three times that with three or more.
            const double rounds = std::ceil((double)blocks / di.cus);
            const double t_mm = rounds * (8.0 + 0.0148 * W->cols);
            const int resident = (int)std::max<size_t>(1, std::min<size_t>(3, (size_t)di.max_lds / xs_bytes(8)));
            const double rate = 1.3e6 * resident;
            const double t_rows = std::max(8.5, 4.0 + std::ceil(batch / 8.0) * (double)W->rows * W->cols / rate);
            const bool take = tu.mfma_min_tokens > 0 ? batch >= tu.mfma_min_tokens : t_mm < t_rows;
            if (take) {
                a.minmax = W->minmax_bf16 ? 1 : 0;
                a.epilogue = 0;
                MmPlan mp;
                mp.smem = mm_lds_bytes(n_order);
                mp.grid = (int)std::min<long long>(units, di.cus);  // a unit per compute unit before a second per compute unit
                return launch_product_mm(a, mp, s);
            }
        }
    }
    const int threads = 256;  // 16 rows at a time
    const long long items = (long long)((batch + tb - 1) / tb) * ((W->rows + threads / 16 - 1) / (threads / 16));
    const int grid = (int)std::min<long long>(items, 8LL * di.cus);
    const size_t smem = xs_bytes(std::max(tb, 4));
    return launch_matvec_rows(a, run, W->minmax_bf16 != nullptr, grid, threads, smem, s);
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
    return launch_decode_dense(a, run, out, grid, static_cast<hipStream_t>(stream));
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
    const size_t smem = decompress_lds_bytes(a.n_order, n_mats);
    if (smem > (size_t)di.max_lds) return QMOE_E_LIMIT;  // (the paper's table leaves room for about 20000 matrices a call)
    // one workgroup per compute unit (its LDS is taken whole); the kernel deals the matrices that have a
    // destination out over them
    const long long total = (long long)n_mats * a.row_blocks;
    const int grid = (int)std::min<long long>(total, (long long)di.cus);
    return launch_decompress(a, out_kind, minmax, grid, smem, static_cast<hipStream_t>(stream));
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
    int lanes_wi = 0, lanes_wo = 0;
    if ((st = split_format(code_order, &code_order, &minmax, &lanes_wi, &lanes_wo)) != QMOE_OK) return st;
    if ((st = check_code_order(d, code_order)) != QMOE_OK) return st;
    const bool run = d->max_nonzeros <= kRunMaxNonzeros;
    const int n_order = code_order ? (int)d->order_table.size() : 0;
    ProductPlan pwi, pwo;
    MmPlan mp;
    const int spread = layer_blocks_hint(n_experts, n_tokens);
    if ((st = plan_product(d_ff, d_model, run, n_tokens, &pwi, n_order,
                           tuning().blocks_first > 0 ? tuning().blocks_first : spread,
                           (d_ff % 8 == 0 && tuning().stage_out >= 0) ? 2 : 0, minmax, lanes_wi)) != QMOE_OK)
        return st;
    if ((st = plan_product(d_model, d_ff, run, n_tokens, &pwo, n_order,
                           tuning().blocks_second > 0 ? tuning().blocks_second : spread,
                           (d_model % 8 == 0 && tuning().stage_out >= 0) ? 4 : 0, minmax, lanes_wo)) != QMOE_OK)
        return st;
    if ((st = plan_mm(d, code_order, d_model, d_ff, n_tokens, true, &mp)) != QMOE_OK) return st;
    return launch_dispatch(expert_idx, n_tokens, n_experts, d_model, layer_ptrs(workspace, l), pwi.tb_max,
                           pwo.tb_max, mp.min_tokens, nullptr, static_cast<hipStream_t>(stream));
}

namespace {

// side: 0 = every kernel on `stream`; 1 = one of the two chains of kernels on `side_stream`, or on the
// library's own second stream when that is NULL
qmoe_status layer_forward(const qmoe_dict *d, const qmoe_matrix *wi, const qmoe_matrix *wo,
                          int code_order, int n_experts, int d_model, int d_ff, const uint16_t *x_bf16,
                          const int32_t *expert_idx, const float *gate, int n_tokens, float *y,
                          void *workspace, size_t workspace_bytes, void *stream, int side, void *side_stream_arg)
{
    qmoe_ws_layout l;
    qmoe_status st = qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens, &l);
    if (st != QMOE_OK) return st;
    if (!d || !wi || !wo || !x_bf16 || !expert_idx || !y) return QMOE_E_INVALID_ARG;
    if (!d->dev) return QMOE_E_NO_DEVICE_DICT;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < l.total)
        return QMOE_E_WORKSPACE;
    bool minmax = false;
    int lanes_wi = 0, lanes_wo = 0;
    if ((st = split_format(code_order, &code_order, &minmax, &lanes_wi, &lanes_wo)) != QMOE_OK) return st;
    if ((st = check_code_order(d, code_order)) != QMOE_OK) return st;
    const bool run = d->max_nonzeros <= kRunMaxNonzeros;
    const int n_order = code_order ? (int)d->order_table.size() : 0;
    ProductPlan pwi, pwo;
    const int spread = layer_blocks_hint(n_experts, n_tokens);
    if ((st = plan_product(d_ff, d_model, run, n_tokens, &pwi, n_order,
                           tuning().blocks_first > 0 ? tuning().blocks_first : spread,
                           (d_ff % 8 == 0 && tuning().stage_out >= 0) ? 2 : 0, minmax, lanes_wi)) != QMOE_OK)
        return st;
    if ((st = plan_product(d_model, d_ff, run, n_tokens, &pwo, n_order,
                           tuning().blocks_second > 0 ? tuning().blocks_second : spread,
                           (d_model % 8 == 0 && tuning().stage_out >= 0) ? 4 : 0, minmax, lanes_wo)) != QMOE_OK)
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
    // With both kinds present one chain goes to a side stream that forks from `stream` after
    // the dispatch and joins it again at the end, so the kernels fill each other's idle compute
    // units; the caller sees the usual stream order.  The chain that stays on `stream` starts
    // first (a kernel behind an event starts several microseconds late) and its persistent
    // workgroups take every compute unit; measured, the step is shorter when that is the SHORTER
    // chain: the longer one then moves in as compute units come free and keeps them to the end,
    // instead of leaving the short chain to run as a thin tail (c2048, where the crowded experts
    // are the short chain: 0.966 against 0.985 ms; 256 experts with 1-32 tokens each, where they
    // are the long one: 1.28 against 1.48 ms).  Limiting each chain to a share of the compute
    // units in proportion to its work was worse than either (measured for shares from 1/4 to 7/8).
    // The host cannot see the routing, so it goes by the average: with four or more tokens per
    // expert most tokens sit in crowded experts.
    const bool overlap = side && mm && tuning().overlap >= 0 && (phases & 6) && (phases & 24);
    const bool mm_first = (long long)n_tokens < 4LL * n_experts;
    hipStream_t s_mm = s, s_sc = s;
    SideStream ss;
    if (overlap) {
        if ((st = side_stream(static_cast<hipStream_t>(side_stream_arg), &ss)) != QMOE_OK) return st;
        if (mm_first) s_sc = ss.stream;
        else s_mm = ss.stream;
        QMOE_HIP_TRY(hipEventRecord(ss.fork, s));
        QMOE_HIP_TRY(hipStreamWaitEvent(ss.stream, ss.fork, 0));
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
    // crowded experts (matrix cores): their tiles are the long items
    if (mm) {
        ProductArgs am = a1;
        am.items = lp.items_mm;
        am.n_items_dev = lp.counters + 7;
        am.work_counter = lp.counters + 8;
        // the hidden vectors of the crowded experts are kept in blocks of 16 tokens (see ProductArgs); only the two
        // matrix-core kernels touch those slots (needs whole 8-column groups on the hidden side: d_ff % 8 == 0)
        am.out_tiled = 1;
        am.mm_in_step = 1;  // its activations come by token rows: the wavefronts of a workgroup read the same lines together
        if (phases & 8)
            if ((st = launch_product_mm(am, mp, s_mm)) != QMOE_OK) return st;
        am = a2;
        am.items = lp.items_mm;
        am.n_items_dev = lp.counters + 7;
        am.work_counter = lp.counters + 9;
        am.x_tiled = 1;
        if (phases & 16)
            if ((st = launch_product_mm(am, mp, s_mm)) != QMOE_OK) return st;
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
        if ((st = launch_product(a1, pwi, run, s_sc)) != QMOE_OK) return st;
    a2.items = lp.items_wo;
    a2.n_items_dev = lp.counters + 4;
    a2.rows_per_item = pwo.rows_per_item;
    a2.blocks_per_pass = pwo.blocks_per_pass;
    a2.tb_max = pwo.tb_max;
    a2.lds_dict_entries = pwo.lds_dict_entries;
    a2.stage_out = pwo.stage_out && reinterpret_cast<uintptr_t>(y) % 16 == 0;
    a2.work_counter = lp.counters + 6;
    if (phases & 4)
        if ((st = launch_product(a2, pwo, run, s_sc)) != QMOE_OK) return st;
    if (overlap) {
        QMOE_HIP_TRY(hipEventRecord(ss.join, ss.stream));
        QMOE_HIP_TRY(hipStreamWaitEvent(s, ss.join, 0));
    }
    return QMOE_OK;
}

}  // namespace

qmoe_status qmoe_moe_layer_forward(const qmoe_dict *d, const qmoe_matrix *wi, const qmoe_matrix *wo,
                                   int code_order, int n_experts, int d_model, int d_ff, const uint16_t *x_bf16,
                                   const int32_t *expert_idx, const float *gate, int n_tokens, float *y,
                                   void *workspace, size_t workspace_bytes, void *stream, void *side_stream)
{
    return layer_forward(d, wi, wo, code_order, n_experts, d_model, d_ff, x_bf16, expert_idx, gate, n_tokens, y,
                         workspace, workspace_bytes, stream, 1, side_stream);
}

int qmoe_plan_lanes(const qmoe_dict *d, int rows, int cols, int n_experts, int n_tokens)
{
    if (!d || rows < 1 || cols < 2 || (cols & 1) || n_experts < 1 || n_tokens < 1 || d->order_table.empty()) return 0;
    ProductPlan p;
    const bool run = d->max_nonzeros <= kRunMaxNonzeros;
    if (plan_product(rows, cols, run, n_tokens, &p, (int)d->order_table.size(), layer_blocks_hint(n_experts, n_tokens)) !=
        QMOE_OK)
        return 0;
    return p.threads * p.blocks_per_pass;
}

size_t qmoe_static_workspace_bytes(void) { return kStaticWsBytes; }

qmoe_status qmoe_moe_layer_forward_static(const qmoe_dict *d, const qmoe_matrix *wi, const qmoe_matrix *wo,
                                          int code_order, int n_experts, int d_model, int d_ff,
                                          const uint16_t *x_bf16, const int32_t *expert_idx, const float *gate,
                                          int n_tokens, float *y, void *stream)
{
    qmoe_ws_layout l;
    const qmoe_status st = qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens, &l);
    if (st != QMOE_OK) return st;
    if (!d || !wi || !wo || !x_bf16 || !expert_idx || !y) return QMOE_E_INVALID_ARG;
    if (!d->dev) return QMOE_E_NO_DEVICE_DICT;
    if (l.total > kStaticWsBytes) return QMOE_E_LIMIT;
    void *ws = nullptr;
    const qmoe_status wst = static_workspace(&ws);
    if (wst != QMOE_OK) return wst;
    // one stream, no events: nothing here creates a stream, an event or memory
    return layer_forward(d, wi, wo, code_order, n_experts, d_model, d_ff, x_bf16, expert_idx, gate, n_tokens, y, ws,
                         kStaticWsBytes, stream, 0, nullptr);
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
    if (phases & 2)
        if ((st = launch_dense_bf16(a, pwi, s)) != QMOE_OK) return st;
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
    if (phases & 4)
        if ((st = launch_dense_bf16(a, pwo, s)) != QMOE_OK) return st;
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
    return launch_renumber(codes, n_codes, map, grid, static_cast<hipStream_t>(stream));
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
    return launch_stream_copy(dst, src, n16, grid, static_cast<hipStream_t>(stream));
}

}  // extern "C"
