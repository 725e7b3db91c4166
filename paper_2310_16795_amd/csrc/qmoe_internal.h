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

// Device blob written by qmoe_dict_upload: run entries first, then the
// interchange-layout words, both for all 65536 codewords (absent entries are 0).
constexpr size_t kDevRunOffset = 0;
constexpr size_t kDevWordsOffset = sizeof(uint32_t) * kTableEntries;
constexpr size_t kDevDictBytes = kDevWordsOffset + 2 * sizeof(uint32_t) * kTableEntries;

struct Tuning {
    int threads = 0;
    int rows_per_item = 0;
    int token_tile = 0;
    int lds_dict_entries = 0;  // 0 = heuristic, -1 = keep the table in L2 only
    int grid_per_cu = 0;
    int host_threads = 0;
    int phases = 0;  // bit 0 dispatch, bit 1 first product, bit 2 second product; 0 = all
};
Tuning &tuning();

}  // namespace qmoe

struct qmoe_dict {
    int n_entries = 0;
    int max_pairs = 0;
    int max_nonzeros = 0;
    std::vector<uint32_t> words;  // [kTableEntries][2], interchange layout, zero beyond n_entries
    std::vector<uint32_t> run;    // [kTableEntries], valid when max_nonzeros <= kRunMaxNonzeros
    // trie over the entries: child[node * 9 + pair] (-1 = none), code[node] (-1 = no entry ends here)
    std::vector<int32_t> child;
    std::vector<int32_t> code;
    const void *dev = nullptr;  // bound by qmoe_dict_upload
};
