// Host side of the library: dictionary generation (Section 4.3.2, Algorithm 1),
// entry layouts, the longest-prefix trie encoder and stream validation
// (Section 4.3.3 "Encoding").  No GPU code in this file.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <map>
#include <queue>
#include <thread>

#include "qmoe_internal.h"
#include "qmoe_hooks.h"

namespace qmoe {

Tuning &tuning()
{
    static Tuning t;
    return t;
}

namespace {

// A candidate sequence of Algorithm 1, symbols packed two bits apiece
// (symbol j at bits 2j..2j+1), plus the counts its probability depends on.
struct Candidate {
    uint64_t syms;   // up to 28 symbols
    uint64_t rank3;  // the symbol string as a base-3 number (first symbol most significant)
    double logp;     // zeros*ln(p0) + nonzeros*ln(q), from the integer counts
    uint8_t npairs, zeros, nonzeros;
};

// priority_queue keeps the element for which "less" is false against all others on top
struct PopsLater {
    bool operator()(const Candidate &a, const Candidate &b) const
    {
        if (a.logp != b.logp) return a.logp < b.logp;
        return a.rank3 > b.rank3;
    }
};

inline int sym_at(uint64_t syms, int j) { return (int)((syms >> (2 * j)) & 3u); }

void pack_words(uint64_t syms, int npairs, uint32_t *w)
{
    // each word: count in the low nibble, then its 14 symbols from bit 4 up
    w[0] = (uint32_t)npairs | (uint32_t)((syms & ((1ull << 28) - 1)) << 4);
    w[1] = (uint32_t)npairs | (uint32_t)(((syms >> 28) & ((1ull << 28) - 1)) << 4);
}

// Device numbering of the codewords: group the sign variants of the last two non-zeros
// of each run under one table entry (see qmoe_internal.h).
// What the two low bits of a device code toggle in its table entry: the sign bits of
// fields 1 and 2.  The kernels apply it to every code; single entries are stored with it
// applied once already.
inline uint32_t order_flips(uint32_t code)
{
    return ((code & 1u) << 18) | ((code & 2u) << 25);
}

void build_device_order(qmoe_dict *d)
{
    d->order_table.clear();
    d->order_map.clear();
    d->n_groups = 0;
    if (d->max_nonzeros > kRunMaxNonzeros) return;
    const int n = d->n_entries;
    struct Nz { int pos; bool neg; };
    // key: run length, positions, and the sign of the first non-zero when there are three
    std::map<std::vector<int>, std::vector<int>> groups;  // key -> member code by free-sign bits, -1 = missing
    std::vector<std::vector<Nz>> nz((size_t)n);
    for (int k = 0; k < n; k++) {
        const uint32_t e = d->run[k];
        for (int j = 0; j < kRunMaxNonzeros; j++) {
            const uint32_t f = (e >> (8 + 8 * j)) & 0xFFu;
            if (f) nz[k].push_back(Nz{(int)(f >> 3), ((f >> 1) & 3u) == 3u});
        }
        const size_t c = nz[k].size();
        if (c < 2) continue;
        std::vector<int> key{(int)(e & 0xFFu)};
        for (const Nz &z : nz[k]) key.push_back(z.pos);
        if (c == 3) key.push_back(nz[k][0].neg ? 1 : 0);
        const int bits = (nz[k][c - 2].neg ? 1 : 0) | (nz[k][c - 1].neg ? 2 : 0);
        std::vector<int> &m = groups[key];
        if (m.empty()) m.assign(4, -1);
        if (m[bits] < 0) m[bits] = k;  // duplicates in a hand-made table stay single entries
    }
    std::vector<uint32_t> table;
    std::vector<int> device_of((size_t)n, -1);
    for (const auto &kv : groups) {
        const std::vector<int> &m = kv.second;
        if (m[0] < 0 || m[1] < 0 || m[2] < 0 || m[3] < 0) continue;
        const int g = (int)table.size();
        const int k = m[0];  // both free signs positive
        const size_t c = nz[k].size();
        uint32_t e = d->run[k] & 0xFFu;
        if (c == 3) e |= (((uint32_t)nz[k][0].pos << 3) | ((nz[k][0].neg ? 3u : 1u) << 1)) << 8;
        e |= (((uint32_t)nz[k][c - 2].pos << 3) | (1u << 1)) << 16;
        e |= (((uint32_t)nz[k][c - 1].pos << 3) | (1u << 1)) << 24;
        table.push_back(e);
        for (int b = 0; b < 4; b++) device_of[m[b]] = 4 * g + b;
    }
    const int n_groups = (int)table.size();
    int next = 4 * n_groups;
    for (int k = 0; k < n; k++) {
        if (device_of[k] >= 0) continue;
        device_of[k] = next++;
        // fields right-aligned like those of the groups: unused ones (0) come first
        uint32_t e = d->run[k];
        while ((e >> 8) != 0u && (e >> 24) == 0u) e = (e & 0xFFu) | ((e & 0xFFFFFF00u) << 8);
        table.push_back(e ^ order_flips((uint32_t)device_of[k]));
    }
    int absent = -1;  // codes that name no entry all map to one empty single entry
    if (n < kTableEntries) {
        absent = next++;
        table.push_back(0u ^ order_flips((uint32_t)absent));
    }
    if ((int)table.size() > kMaxOrderTable || next > kTableEntries) return;
    d->order_map.assign(kTableEntries, (uint16_t)(absent >= 0 ? absent : 0));
    for (int k = 0; k < n; k++) d->order_map[k] = (uint16_t)device_of[k];
    d->order_table = std::move(table);
    d->n_groups = n_groups;
}

// Derive everything the codec and the kernels need from the interchange words.
qmoe_status finish_dict(qmoe_dict *d)
{
    const int n = d->n_entries;
    d->run.assign(kTableEntries, 0u);
    d->max_nonzeros = 0;
    d->max_pairs = 0;
    for (int k = 0; k < n; k++) {
        const uint32_t w0 = d->words[2 * k], w1 = d->words[2 * k + 1];
        const int np = (int)(w0 & 15u);
        if (np < 1 || np > 14 || (int)(w1 & 15u) != np) return QMOE_E_BAD_SYMBOL;
        d->max_pairs = std::max(d->max_pairs, np);
        uint32_t run = (uint32_t)(8 * 2 * np);
        int nnz = 0;
        for (int j = 0; j < kMaxSyms; j++) {
            const uint32_t w = j < 14 ? w0 : w1;
            const int s = (int)((w >> (4 + 2 * (j % 14))) & 3u);
            if (s == 3) return QMOE_E_BAD_SYMBOL;
            if (j >= 2 * np && s != 0) return QMOE_E_BAD_SYMBOL;
            if (s != 0) {
                if (nnz < kRunMaxNonzeros) {
                    const uint32_t weight = (s == 2) ? 1u : 3u;  // 2-bit signed: +1 / -1
                    run |= (((uint32_t)j << 3) | (weight << 1)) << (8 + 8 * nnz);
                }
                nnz++;
            }
        }
        d->max_nonzeros = std::max(d->max_nonzeros, nnz);
        d->run[k] = run;
    }
    build_device_order(d);
    // trie: node 0 is the root; an entry's node is reached by its pairs in order
    d->child.assign(9, -1);
    d->code.assign(1, -1);
    for (int k = 0; k < n; k++) {
        const uint32_t w0 = d->words[2 * k], w1 = d->words[2 * k + 1];
        const int np = (int)(w0 & 15u);
        int node = 0;
        for (int j = 0; j < np; j++) {
            const uint32_t w = j < 7 ? w0 : w1;
            const int pr = (int)((w >> (4 + 4 * (j % 7))) & 15u);  // two symbols = 4 bits
            const int pair = 3 * (pr & 3) + (pr >> 2);             // first symbol is the low one
            int nx = d->child[(size_t)node * 9 + pair];
            if (nx < 0) {
                nx = (int)d->code.size();
                d->code.push_back(-1);
                d->child.resize(d->child.size() + 9, -1);
                d->child[(size_t)node * 9 + pair] = nx;
            }
            node = nx;
        }
        if (d->code[node] < 0) d->code[node] = k;  // duplicates: the earlier (more probable) index wins
    }
    return QMOE_OK;
}

inline int pair_of(int8_t a, int8_t b)
{
    // value -> symbol: 0 -> 0, -1 -> 1, +1 -> 2 ; returns -1 for anything else
    const int sa = a == 0 ? 0 : (a == -1 ? 1 : (a == 1 ? 2 : -1));
    const int sb = b == 0 ? 0 : (b == -1 ? 1 : (b == 1 ? 2 : -1));
    return (sa < 0 || sb < 0) ? -1 : 3 * sa + sb;
}

// Encode rows [r0, r1) into out (appended), counts[r - r0] = codewords of row r.
qmoe_status encode_rows(const qmoe_dict *d, const int8_t *tern, int cols, int r0, int r1,
                        std::vector<uint16_t> *out, uint32_t *counts, bool store)
{
    const int32_t *child = d->child.data();
    const int32_t *code = d->code.data();
    const int np = cols / 2;
    for (int r = r0; r < r1; r++) {
        const int8_t *row = tern + (size_t)r * cols;
        uint32_t n = 0;
        int i = 0;
        while (i < np) {
            int node = 0, best = -1, best_len = 0, depth = 0;
            while (i + depth < np) {
                const int pr = pair_of(row[2 * (i + depth)], row[2 * (i + depth) + 1]);
                if (pr < 0) return QMOE_E_BAD_SYMBOL;
                const int nx = child[(size_t)node * 9 + pr];
                if (nx < 0) break;
                node = nx;
                depth++;
                if (code[node] >= 0) {
                    best = code[node];
                    best_len = depth;
                }
            }
            if (best < 0) return QMOE_E_UNENCODABLE;
            if (store) out->push_back((uint16_t)best);
            n++;
            i += best_len;
        }
        counts[r - r0] = n;
    }
    return QMOE_OK;
}

}  // namespace
}  // namespace qmoe

using namespace qmoe;

extern "C" {

const char *qmoe_strerror(qmoe_status s)
{
    switch (s) {
    case QMOE_OK: return "ok";
    case QMOE_E_INVALID_ARG: return "invalid argument";
    case QMOE_E_BUFFER_TOO_SMALL: return "output buffer too small";
    case QMOE_E_BAD_SYMBOL: return "symbol outside the ternary alphabet";
    case QMOE_E_CORRUPT_STREAM: return "corrupt codeword stream";
    case QMOE_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case QMOE_E_HIP: return "HIP call failed";
    case QMOE_E_UNENCODABLE: return "input not encodable with this dictionary";
    case QMOE_E_NOMEM: return "out of host memory";
    case QMOE_E_NO_DEVICE_DICT: return "dictionary not uploaded to the device";
    case QMOE_E_LIMIT: return "size beyond the supported limit";
    default: return "unknown status";
    }
}

qmoe_status qmoe_dict_create(double p0, int max_pairs, int n_entries, qmoe_dict **out)
{
    if (!out || !(p0 > 0.0 && p0 < 1.0) || max_pairs < 1 || max_pairs > 14 || n_entries < 1 ||
        n_entries > kTableEntries)
        return QMOE_E_INVALID_ARG;
    *out = nullptr;
    qmoe_dict *d = new (std::nothrow) qmoe_dict;
    if (!d) return QMOE_E_NOMEM;
    try {
        d->words.assign(2 * (size_t)kTableEntries, 0u);
        const double lp0 = std::log(p0), lq = std::log((1.0 - p0) / 2.0);
        std::priority_queue<Candidate, std::vector<Candidate>, PopsLater> queue;
        queue.push(Candidate{0, 0, 0.0, 0, 0, 0});
        int count = 0;
        while (count < n_entries && !queue.empty()) {
            const Candidate s = queue.top();
            queue.pop();
            if (s.npairs >= 1) {  // never above max_pairs: such candidates are not queued
                pack_words(s.syms, s.npairs, &d->words[2 * (size_t)count]);
                count++;
            }
            if (s.npairs == max_pairs) continue;  // longer sequences can never be appended
            for (int t1 = 0; t1 < 3; t1++)
                for (int t2 = 0; t2 < 3; t2++) {
                    Candidate c = s;
                    c.syms |= ((uint64_t)t1 | ((uint64_t)t2 << 2)) << (4 * s.npairs);
                    c.rank3 = s.rank3 * 9 + (uint64_t)(3 * t1 + t2);
                    c.npairs = (uint8_t)(s.npairs + 1);
                    c.zeros = (uint8_t)(s.zeros + (t1 == 0) + (t2 == 0));
                    c.nonzeros = (uint8_t)(s.nonzeros + (t1 != 0) + (t2 != 0));
                    c.logp = (double)c.zeros * lp0 + (double)c.nonzeros * lq;
                    queue.push(c);
                }
        }
        d->n_entries = count;
        const qmoe_status st = finish_dict(d);
        if (st != QMOE_OK) {
            delete d;
            return st;
        }
    } catch (const std::bad_alloc &) {
        delete d;
        return QMOE_E_NOMEM;
    }
    *out = d;
    return QMOE_OK;
}

qmoe_status qmoe_dict_from_words(const uint32_t *words, int n_entries, qmoe_dict **out)
{
    if (!out || !words || n_entries < 1 || n_entries > kTableEntries) return QMOE_E_INVALID_ARG;
    *out = nullptr;
    qmoe_dict *d = new (std::nothrow) qmoe_dict;
    if (!d) return QMOE_E_NOMEM;
    try {
        d->words.assign(2 * (size_t)kTableEntries, 0u);
        std::memcpy(d->words.data(), words, 2 * sizeof(uint32_t) * (size_t)n_entries);
        d->n_entries = n_entries;
        const qmoe_status st = finish_dict(d);
        if (st != QMOE_OK) {
            delete d;
            return st;
        }
    } catch (const std::bad_alloc &) {
        delete d;
        return QMOE_E_NOMEM;
    }
    *out = d;
    return QMOE_OK;
}

qmoe_status qmoe_dict_words(const qmoe_dict *d, const uint32_t **words, int *n_entries)
{
    if (!d || !words || !n_entries) return QMOE_E_INVALID_ARG;
    *words = d->words.data();
    *n_entries = d->n_entries;
    return QMOE_OK;
}

int qmoe_dict_max_nonzeros(const qmoe_dict *d) { return d ? d->max_nonzeros : QMOE_E_INVALID_ARG; }

size_t qmoe_dict_device_bytes(void) { return kDevDictBytes; }

qmoe_status qmoe_dict_device_order(const qmoe_dict *d, const uint16_t **code_map, const uint32_t **table,
                                   int *n_groups, int *n_table)
{
    if (!d || !code_map || !table || !n_groups || !n_table) return QMOE_E_INVALID_ARG;
    *code_map = d->order_map.empty() ? nullptr : d->order_map.data();
    *table = d->order_table.empty() ? nullptr : d->order_table.data();
    *n_groups = d->n_groups;
    *n_table = (int)d->order_table.size();
    return QMOE_OK;
}

void qmoe_dict_destroy(qmoe_dict *d) { delete d; }

qmoe_status qmoe_encode_host(const qmoe_dict *d, const int8_t *tern, int rows, int cols, uint16_t *codes,
                             size_t codes_cap, uint32_t *row_off, size_t *n_codes)
{
    if (!d || !tern || !row_off || !n_codes || rows < 1 || cols < 2 || (cols & 1))
        return QMOE_E_INVALID_ARG;
    int nthreads = tuning().host_threads;
    if (nthreads <= 0) {
        if (const char *env = std::getenv("QMOE_HOST_THREADS")) nthreads = std::atoi(env);
        if (nthreads <= 0) nthreads = (int)std::min(16u, std::max(1u, std::thread::hardware_concurrency()));
    }
    nthreads = std::max(1, std::min(nthreads, (rows + 63) / 64));
    try {
        std::vector<uint32_t> counts((size_t)rows);
        std::vector<std::vector<uint16_t>> local((size_t)nthreads);
        std::vector<qmoe_status> status((size_t)nthreads, QMOE_OK);
        auto work = [&](int t) {
            const int r0 = (int)((int64_t)rows * t / nthreads), r1 = (int)((int64_t)rows * (t + 1) / nthreads);
            if (codes) local[t].reserve((size_t)(r1 - r0) * (size_t)(cols / 16 + 4));
            try {
                status[t] = encode_rows(d, tern, cols, r0, r1, &local[t], counts.data() + r0, codes != nullptr);
            } catch (const std::bad_alloc &) {
                status[t] = QMOE_E_NOMEM;
            }
        };
        if (nthreads == 1) {
            work(0);
        } else {
            std::vector<std::thread> pool;
            for (int t = 0; t < nthreads; t++) pool.emplace_back(work, t);
            for (auto &th : pool) th.join();
        }
        for (int t = 0; t < nthreads; t++)
            if (status[t] != QMOE_OK) return status[t];
        uint64_t total = 0;
        for (int r = 0; r < rows; r++) {
            row_off[r] = (uint32_t)total;
            total += counts[r];
        }
        if (total > 0xFFFFFFFFull) return QMOE_E_LIMIT;
        row_off[rows] = (uint32_t)total;
        *n_codes = (size_t)total;
        if (!codes) return QMOE_OK;
        if (codes_cap < total) return QMOE_E_BUFFER_TOO_SMALL;
        for (int t = 0; t < nthreads; t++) {
            const int r0 = (int)((int64_t)rows * t / nthreads);
            if (!local[t].empty())
                std::memcpy(codes + row_off[r0], local[t].data(), local[t].size() * sizeof(uint16_t));
        }
    } catch (const std::bad_alloc &) {
        return QMOE_E_NOMEM;
    }
    return QMOE_OK;
}

qmoe_status qmoe_validate_host(const qmoe_dict *d, const uint16_t *codes, const uint32_t *row_off, int rows,
                               int cols)
{
    if (!d || !codes || !row_off || rows < 1 || cols < 2 || (cols & 1)) return QMOE_E_INVALID_ARG;
    if (row_off[0] != 0) return QMOE_E_CORRUPT_STREAM;
    for (int r = 0; r < rows; r++) {
        if (row_off[r + 1] < row_off[r]) return QMOE_E_CORRUPT_STREAM;
        int64_t idx = 0;
        for (uint32_t k = row_off[r]; k < row_off[r + 1]; k++) {
            const uint32_t c = codes[k];
            if ((int)c >= d->n_entries) return QMOE_E_CORRUPT_STREAM;
            idx += 2 * (int64_t)(d->words[2 * (size_t)c] & 15u);
            if (idx > cols) return QMOE_E_CORRUPT_STREAM;
        }
        if (idx != cols) return QMOE_E_CORRUPT_STREAM;
    }
    return QMOE_OK;
}

// ---- lane-interleaved device layout of a codeword stream (see include/qmoe.h) ----
namespace {

// rows [*ra, *rb) of lane g when `rows` rows are dealt evenly over `lanes` lanes
inline void lane_rows(int rows, int lanes, int g, int *ra, int *rb)
{
    const int base = rows / lanes, extra = rows - base * lanes;
    *ra = g * base + std::min(g, extra);
    *rb = *ra + base + (g < extra ? 1 : 0);
}

qmoe_status lane_layout_walk(const uint32_t *row_off, int rows, int lanes, uint32_t *wave_off, size_t *n_pieces)
{
    if (!row_off || rows < 1 || lanes < 64 || (lanes % 64) || lanes > 16320) return QMOE_E_INVALID_ARG;
    unsigned long long total = 0;
    for (int w = 0; w < lanes / 64; w++) {
        if (wave_off) wave_off[w] = (uint32_t)total;
        uint32_t most = 0;
        for (int g = 64 * w; g < 64 * w + 64; g++) {
            int ra, rb;
            lane_rows(rows, lanes, g, &ra, &rb);
            if (row_off[rb] < row_off[ra]) return QMOE_E_CORRUPT_STREAM;
            most = std::max(most, (row_off[rb] - row_off[ra] + 7u) / 8u);
        }
        total += 64ull * most;
        if (total > 0xFFFFFFFFull) return QMOE_E_LIMIT;
    }
    if (wave_off) wave_off[lanes / 64] = (uint32_t)total;
    *n_pieces = (size_t)total;
    return QMOE_OK;
}

}  // namespace

qmoe_status qmoe_lane_layout_size(const uint32_t *row_off, int rows, int lanes, size_t *n_pieces)
{
    if (!n_pieces) return QMOE_E_INVALID_ARG;
    return lane_layout_walk(row_off, rows, lanes, nullptr, n_pieces);
}

qmoe_status qmoe_lane_layout_build(const uint16_t *codes, const uint32_t *row_off, int rows, int lanes, uint16_t *out,
                                   size_t out_pieces, uint32_t *wave_off)
{
    if (!codes || !out || !wave_off) return QMOE_E_INVALID_ARG;
    size_t need = 0;
    const qmoe_status st = lane_layout_walk(row_off, rows, lanes, wave_off, &need);
    if (st != QMOE_OK) return st;
    if (out_pieces < need) return QMOE_E_BUFFER_TOO_SMALL;
    std::memset(out, 0, 16 * need);
    for (int g = 0; g < lanes; g++) {
        int ra, rb;
        lane_rows(rows, lanes, g, &ra, &rb);
        const uint32_t k0 = row_off[ra], n = row_off[rb] - k0;
        const size_t first = (size_t)wave_off[g / 64] + (size_t)(g % 64);  // piece p of the lane sits at first + 64 p
        for (uint32_t i = 0; i < n; i++) out[8 * (first + 64 * (size_t)(i / 8)) + (i % 8)] = codes[k0 + i];
    }
    return QMOE_OK;
}

qmoe_status qmoe_lane_layout_unpack(const uint16_t *pieces, const uint32_t *wave_off, const uint32_t *row_off, int rows,
                                    int lanes, uint16_t *codes, size_t codes_cap)
{
    if (!pieces || !wave_off || !row_off || !codes || rows < 1 || lanes < 64 || (lanes % 64)) return QMOE_E_INVALID_ARG;
    if (codes_cap < row_off[rows]) return QMOE_E_BUFFER_TOO_SMALL;
    for (int g = 0; g < lanes; g++) {
        int ra, rb;
        lane_rows(rows, lanes, g, &ra, &rb);
        const uint32_t k0 = row_off[ra], n = row_off[rb] - k0;
        const size_t first = (size_t)wave_off[g / 64] + (size_t)(g % 64);
        for (uint32_t i = 0; i < n; i++) codes[k0 + i] = pieces[8 * (first + 64 * (size_t)(i / 8)) + (i % 8)];
    }
    return QMOE_OK;
}

qmoe_status qmoe_set_tuning(const char *key, int value)
{
    if (!key) return QMOE_E_INVALID_ARG;
    Tuning &t = tuning();
    if (!std::strcmp(key, "threads")) t.threads = value;
    else if (!std::strcmp(key, "rows_per_item")) t.rows_per_item = value;
    else if (!std::strcmp(key, "token_tile")) t.token_tile = value;
    else if (!std::strcmp(key, "lds_dict_entries")) t.lds_dict_entries = value;
    else if (!std::strcmp(key, "grid_per_cu")) t.grid_per_cu = value;
    else if (!std::strcmp(key, "host_threads")) t.host_threads = value;
    else if (!std::strcmp(key, "blocks_first")) t.blocks_first = value;
    else if (!std::strcmp(key, "blocks_second")) t.blocks_second = value;
    else if (!std::strcmp(key, "mfma_min_tokens")) t.mfma_min_tokens = value;
    else if (!std::strcmp(key, "overlap")) t.overlap = value;
    else return QMOE_E_INVALID_ARG;
    return QMOE_OK;
}

qmoe_status qmoe_hook_set(const char *key, int value)
{
    if (!key) return QMOE_E_INVALID_ARG;
    Tuning &t = tuning();
    if (!std::strcmp(key, "phases")) t.phases = value;
    else if (!std::strcmp(key, "stage_out")) t.stage_out = value;
    else return QMOE_E_INVALID_ARG;
    return QMOE_OK;
}

}  // extern "C"
