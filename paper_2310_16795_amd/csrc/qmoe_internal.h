// Internal declarations shared by the host codec and the HIP launch code.
// Not part of the C ABI.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "qmoe.h"

namespace qmoe {

constexpr int kMaxSyms = 28;          // 14 pairs, two ternary symbols each
constexpr int kTableEntries = 65536;  // device tables always span every uint16 codeword

// Compact device entry ("run entry") for tables whose entries hold at most three
// non-zero symbols, which is the case for the paper's table: a codeword is then
// a run length plus at most three signed positions.  Four bytes:
//   byte 0        8 * (number of ternary values the entry decodes to), 16..224; 0 = no entry
//   byte 1+j      field of the j-th non-zero (j = 0,1,2), 0 = slot unused:
//                   bit 0      always 0
//                   bits 1..2  its weight as a 2-bit signed integer: +1 (01) or -1 (11)
//                   bits 3..7  its position inside the run
// The product kernel keeps one token's activations as 8-byte records {0, +x, 0, -x}
// (bf16) per column: byte 0 is then the distance in bytes the decoder advances, and a
// field is the byte offset, from the record of the run's first column, of the value
// to add -- unused fields land on a zero.
constexpr int kRunMaxNonzeros = 3;

// Device numbering of the codewords ("device order").  The table is small enough to
// sit in LDS whole when sign variants share an entry: codewords are renumbered so that
// four consecutive device codes 4g..4g+3 are the four sign combinations of the last two
// non-zeros of one run (its first non-zero, if it has three, keeps a fixed sign), and
// their common entry is table[g] with those two signs positive; the two low code bits
// then flip the sign bits of fields 1 and 2.  Entries that have no complete group of
// four (at most one non-zero, or variants missing from the dictionary) follow as
// "single" codes, device code = 4 * n_groups + i, entry table[n_groups + i], stored with the
// flips of its own code's two low bits applied (a kernel flips every code alike and so
// restores them).  A stream is
// rewritten once, in place, when it is loaded; its length and the set of runs it can
// express are unchanged.
constexpr int kMaxOrderTable = 20480;  // entries (80 KiB); larger tables keep the interchange numbering

// Device blob written by qmoe_dict_upload: run entries, then the interchange-layout
// words, both for all 65536 codewords (absent entries are 0), then the device-order
// table (kMaxOrderTable entries) and the interchange -> device code map (65536 x u16).
constexpr size_t kDevRunOffset = 0;
constexpr size_t kDevWordsOffset = sizeof(uint32_t) * kTableEntries;
constexpr size_t kDevOrderTableOffset = kDevWordsOffset + 2 * sizeof(uint32_t) * kTableEntries;
constexpr size_t kDevOrderMapOffset = kDevOrderTableOffset + sizeof(uint32_t) * kMaxOrderTable;
// ... then the encoder's trie for qmoe_encode_device: child[node][9] (next node by pair, -1 =
// none; node 0 is the root) and code[node] (codeword that ends here, -1 = none).  A
// prefix-closed table (the paper's is) has n_entries + 1 nodes; tables with more than
// kMaxTrieNodes nodes cannot be used by the device encoder.
constexpr int kMaxTrieNodes = 1 << 17;
constexpr size_t kDevTrieChildOffset = (kDevOrderMapOffset + sizeof(uint16_t) * kTableEntries + 255) / 256 * 256;
constexpr size_t kDevTrieCodeOffset = kDevTrieChildOffset + sizeof(int32_t) * 9 * kMaxTrieNodes;
constexpr size_t kDevDictBytes = kDevTrieCodeOffset + sizeof(int32_t) * kMaxTrieNodes;

struct Tuning {
    int threads = 0;
    int rows_per_item = 0;
    int token_tile = 0;
    int lds_dict_entries = 0;  // 0 = heuristic, -1 = keep the table in L2 only
    int grid_per_cu = 0;
    int host_threads = 0;
    int blocks_first = 0;   // forced blocks per matrix pass, first / single product
    int blocks_second = 0;  // same, second product of a layer
    int stage_out = 0;  // -1 = the first product writes its hidden values straight to global memory
    int overlap = 0;  // -1 = all kernels of a layer on the caller's stream, one after the other
    int mfma_min_tokens = 0;  // 0 = heuristic, -1 = never use the matrix-core kernel
    int phases = 0;  // kernels of a layer call to enqueue: bit 0 dispatch, bits 1 / 2 scalar kernel of the first / second
                     // product, bits 3 / 4 matrix-core kernel of the first / second product; 0 = all
};
Tuning &tuning();

}  // namespace qmoe

struct qmoe_dict {
    int n_entries = 0;
    int max_pairs = 0;
    int max_nonzeros = 0;
    std::vector<uint32_t> words;  // [kTableEntries][2], interchange layout, zero beyond n_entries
    std::vector<uint32_t> run;    // [kTableEntries], valid when max_nonzeros <= kRunMaxNonzeros
    // device order (empty when the dictionary does not qualify)
    std::vector<uint32_t> order_table;  // n_groups group entries, then the single entries
    std::vector<uint16_t> order_map;    // [kTableEntries] interchange code -> device code
    int n_groups = 0;
    // trie over the entries: child[node * 9 + pair] (-1 = none), code[node] (-1 = no entry ends here)
    std::vector<int32_t> child;
    std::vector<int32_t> code;
    const void *dev = nullptr;  // bound by qmoe_dict_upload
};
