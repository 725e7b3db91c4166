/*
 * qmoe.h -- C ABI of the compressed-MoE inference hot path for AMD MI355X (gfx950).
 *
 * The library implements the inference side of QMoE (arxiv 2310.16795,
 * Section 4.3): expert weight matrices are ternary ({-s, 0, +s} with one
 * scale per output row), stored as a stream of 16-bit codewords that index a
 * static dictionary of variable-length ternary runs, and are multiplied with
 * the tokens routed to the expert while being decoded on the fly.
 *
 * Conventions
 *  - A matrix is [rows = output features][cols = input features]; every row is
 *    an independent codeword stream (Section 4.3.1), rows are packed back to
 *    back, row_off[r] is the index (in codewords) of row r's first codeword and
 *    row_off[rows] the total (Section 4.3.3 "Encoding").
 *  - Ternary symbols: 0 -> 0, 1 -> -s_r (the paper's w_min), 2 -> +s_r (w_max).
 *  - "host" / "device" after a pointer says where the memory must live.  The
 *    library never allocates or frees device memory and never synchronises:
 *    device work is enqueued on the caller's stream (a hipStream_t passed as
 *    void*, NULL = the default stream) and the call returns at once.
 *  - Every function returns QMOE_OK or a negative qmoe_status.  Argument
 *    errors are found before anything is enqueued.  The contents of device
 *    buffers are trusted: a corrupt codeword stream is not detected on the
 *    device (run qmoe_validate_host on the host copy first); the kernels clamp
 *    the row offsets to n_codes and every table index and column they derive from a
 *    codeword, so such a stream gives wrong numbers, not an access outside the
 *    buffers described here.
 *  - Nothing crosses the boundary but plain pointers, sizes and the opaque
 *    qmoe_dict handle.
 *  - Process-wide state: the last HIP error code; the launch tuning
 *    (qmoe_set_tuning); per device, created on first use and kept until the process
 *    ends: the device's compute-unit count and LDS size, two events and -- only if a
 *    layer call brings no second stream of its own -- one stream (qmoe_moe_layer_forward),
 *    and the address of the 8 MiB scratch array of qmoe_moe_layer_forward_static.
 */
#ifndef QMOE_H
#define QMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int qmoe_status;
#define QMOE_OK 0
#define QMOE_E_INVALID_ARG (-1)      /* NULL pointer, non-positive size, odd cols, ... */
#define QMOE_E_BUFFER_TOO_SMALL (-2) /* output capacity too small; the needed size is reported */
#define QMOE_E_BAD_SYMBOL (-3)       /* ternary input outside {-1,0,+1}, or symbol value 3 in a table */
#define QMOE_E_CORRUPT_STREAM (-4)   /* a row does not decode to exactly cols values, bad offsets */
#define QMOE_E_WORKSPACE (-5)        /* workspace missing, misaligned or too small */
#define QMOE_E_HIP (-6)              /* a HIP call failed; see qmoe_last_hip_error() */
#define QMOE_E_UNENCODABLE (-7)      /* the dictionary lacks a phrase needed for this input */
#define QMOE_E_NOMEM (-8)            /* host allocation failed */
#define QMOE_E_NO_DEVICE_DICT (-9)   /* device call before qmoe_dict_upload */
#define QMOE_E_LIMIT (-10)           /* size beyond what the kernels support (see each call) */

const char *qmoe_strerror(qmoe_status s);
/* hipError_t of the most recent failed HIP call made by this library (0 = none). */
int qmoe_last_hip_error(void);

/* ------------------------------------------------------------------------- */
/* Dictionary (Section 4.3.2, Algorithm 1)                                    */
/* ------------------------------------------------------------------------- */

typedef struct qmoe_dict qmoe_dict; /* host object; immutable after upload; caller destroys */

/*
 * Generate the static dictionary: the n_entries most probable sequences of
 * 1..max_pairs pairs of ternary symbols under P(0)=p0, P(1)=P(2)=(1-p0)/2
 * (Eq. 2), in order of decreasing probability; equally probable sequences in
 * ascending order of the symbol string read as a base-3 number.  The paper's
 * table is p0 = 0.885, max_pairs = 14, n_entries = 65536.
 * Errors: INVALID_ARG unless 0<p0<1, 1<=max_pairs<=14, 1<=n_entries<=65536.
 * Fewer than n_entries are produced when fewer sequences exist.
 */
qmoe_status qmoe_dict_create(double p0, int max_pairs, int n_entries, qmoe_dict **out);

/*
 * Adopt a table in the interchange layout (host, copied): words[2k], words[2k+1]
 * describe entry k; in each 32-bit word bits 0..3 hold the entry's pair count
 * (the same in both words) and bits 4+2j..5+2j the j-th symbol of that half
 * (7 pairs = 14 symbols per word, first half in word 0), unused slots 0
 * (Section 4.3.2; bit positions as the paper's kernel listing reads them).
 * Errors: INVALID_ARG, BAD_SYMBOL (a symbol value 3, a non-zero unused slot,
 * count nibbles that differ or are 0 or > 14).
 */
qmoe_status qmoe_dict_from_words(const uint32_t *words /*host [n_entries][2]*/, int n_entries,
                                 qmoe_dict **out);

/* Borrow the interchange-layout table (valid until qmoe_dict_destroy). */
qmoe_status qmoe_dict_words(const qmoe_dict *d, const uint32_t **words, int *n_entries);

/* Largest number of non-zero symbols in any entry (3 for the paper's table). */
int qmoe_dict_max_nonzeros(const qmoe_dict *d);

/* Bytes of device memory qmoe_dict_upload needs (independent of the table's contents). */
size_t qmoe_dict_device_bytes(void);

/*
 * The device numbering of the codewords ("device order"), for dictionaries whose
 * entries hold at most three non-zeros.  The paper keeps its table in L2 and notes
 * that look-ups are random accesses (Section 4.3.2); to hold the whole table in the
 * 160 KB of LDS instead, this library renumbers the codewords so that the four sign
 * combinations of the last two non-zeros of a run are four consecutive codes
 * 4g..4g+3 sharing one table entry; runs without a complete group of four follow as
 * single codes.  It is a bijection on the codes in use: stream length, bits per
 * parameter and the set of runs are unchanged.
 *   code_map [65536]   interchange code -> device code
 *   table    [n_table] entry of group g at table[g] (both free signs positive), entry of
 *                      single code c = 4*n_groups + i at table[n_groups + i], stored with the
 *                      toggles of c's own two low bits (below) applied; each entry is
 *                      byte 0 = 8 * run length, bytes 1..3 = one field per non-zero:
 *                      (position << 3) | (weight as 2-bit signed integer << 1), 0 = unused;
 *                      the fields are right-aligned (k non-zeros fill bytes 4-k..3 in
 *                      ascending position), so unused fields always come first
 * Device code c decodes to table[c < 4*n_groups ? c >> 2 : c - 3*n_groups] with bit 2 of
 * field 1 toggled if c & 1 and bit 2 of field 2 toggled if c & 2 (in a group that turns
 * weight +1 into -1; for a single code it undoes the stored toggles), so a kernel treats
 * every code alike.
 * code_map and table are NULL (n_table = 0) when the dictionary has no device order.
 */
qmoe_status qmoe_dict_device_order(const qmoe_dict *d, const uint16_t **code_map, const uint32_t **table,
                                   int *n_groups, int *n_table);

/*
 * Copy the device form of the table into dev_buf (device, >= qmoe_dict_device_bytes(),
 * 256-byte aligned, owned by the caller, must outlive every device call that uses d)
 * and bind it to d.  The copy is enqueued on `stream` from memory owned by d.
 * Errors: INVALID_ARG, BUFFER_TOO_SMALL, HIP.
 */
qmoe_status qmoe_dict_upload(qmoe_dict *d, void *dev_buf /*device*/, size_t dev_bytes, void *stream);

void qmoe_dict_destroy(qmoe_dict *d);

/* ------------------------------------------------------------------------- */
/* Host codec (Section 4.3.3 "Encoding")                                      */
/* ------------------------------------------------------------------------- */

/*
 * Encode a row-major ternary matrix (host int8 in {-1,0,+1}) by longest-prefix
 * match against the dictionary, row by row.  row_off (host, [rows+1]) is always
 * written; codes (host) may be NULL to only size the output.  *n_codes receives
 * the number of codewords needed.  Rows are encoded on several host threads.
 * Errors: INVALID_ARG (NULL, rows<1, cols<2 or odd), BAD_SYMBOL,
 * BUFFER_TOO_SMALL (codes_cap < needed; *n_codes still set), UNENCODABLE,
 * LIMIT (more than 2^32-1 codewords).
 */
qmoe_status qmoe_encode_host(const qmoe_dict *d, const int8_t *tern /*host [rows][cols]*/, int rows,
                             int cols, uint16_t *codes /*host or NULL*/, size_t codes_cap,
                             uint32_t *row_off /*host [rows+1]*/, size_t *n_codes);

/*
 * Check a compressed matrix on the host: offsets start at 0 and never decrease,
 * every codeword names an entry, every row decodes to exactly cols values.
 * Errors: INVALID_ARG, CORRUPT_STREAM.
 */
qmoe_status qmoe_validate_host(const qmoe_dict *d, const uint16_t *codes /*host*/,
                               const uint32_t *row_off /*host [rows+1]*/, int rows, int cols);

/*
 * The same encoder on the device (Section 4.3.3 "Encoding"), one matrix row per lane:
 * ternary (device, row-major int8 [rows][cols], values -1/0/+1) is coded into codes
 * (device, capacity codes_cap codewords, interchange numbering -- run
 * qmoe_codes_to_device_order on it afterwards for the device numbering) and row_off
 * (device [rows+1]); row_off[rows] is the number of codewords.  Codeword for codeword the
 * stream qmoe_encode_host produces.  Nothing is read back: status (device int32[2]) holds
 * 0 or the first error (BAD_SYMBOL, UNENCODABLE, BUFFER_TOO_SMALL) and a row it happened
 * in once the work on `stream` is done; with an error the contents of codes are
 * undefined.  Enqueues four kernels (the first clears status), no memset.
 * Errors at the call: INVALID_ARG, NO_DEVICE_DICT, LIMIT (the table's trie has more than
 * 131072 nodes), HIP.
 */
qmoe_status qmoe_encode_device(const qmoe_dict *d, const int8_t *ternary /*device*/, int rows, int cols,
                               uint16_t *codes /*device*/, size_t codes_cap, uint32_t *row_off /*device*/,
                               int32_t *status /*device*/, void *stream);

/* ------------------------------------------------------------------------- */
/* Device kernels (Section 4.3.3 "GPU Kernel")                                */
/* ------------------------------------------------------------------------- */

/*
 * One compressed matrix.  All pointers are device memory owned by the caller.
 * The grid of a row is {-s_r, 0, +s_r} with s_r = scale_f16[r] (symbol 1 = -s_r, symbol 2 =
 * +s_r), or, when minmax_bf16 is not NULL, the asymmetric {w_min, 0, w_max} of Section 4.1
 * with one bfloat16 pair per row as in Listing 1 (symbol 1 = w_min, symbol 2 = w_max,
 * "Ternary decoding" in Section 4.3.3; either may have any sign); scale_f16 is not read then.
 */
typedef struct qmoe_matrix {
    const uint16_t *codes;     /* [n_codes] codewords, rows back to back; 16-byte aligned,
                                  readable (any contents) up to the next 16-byte
                                  boundary after the last codeword                      */
    const uint32_t *row_off;   /* [rows+1] first codeword of each row                   */
    const uint16_t *scale_f16; /* [rows] IEEE binary16 scale s_r of each output row     */
    int32_t rows, cols;        /* cols even                                             */
    uint32_t n_codes;          /* = row_off[rows]; offsets beyond it are clamped        */
    uint32_t code_order;       /* 0: interchange numbering (as encoded); 1: device
                                  numbering (after qmoe_codes_to_device_order)          */
    const uint16_t *minmax_bf16; /* NULL, or [rows][2] bfloat16 (w_min, w_max) of each
                                  output row, 4-byte aligned                            */
    const uint32_t *wave_off;  /* lane-interleaved layout (below): [lanes/64 + 1] first
                                  16-byte piece of each group of 64 lanes; else NULL     */
    uint32_t lanes;            /* lane-interleaved layout: the lane count it was built
                                  for; 0 = rows back to back (the interchange layout)   */
    uint32_t reserved;         /* 0 */
} qmoe_matrix;

/*
 * Lane-interleaved device layout of a stream (a load-time re-packing, like the device
 * numbering; the paper's kernel reads 32 consecutive codewords of one row with one coalesced
 * transaction, Section 4.3.3 "Execution" -- this is the same for a kernel that gives every
 * lane a row range of its own).  The rows of a matrix are dealt evenly over `lanes` lanes
 * (lane g owns rows g*b + min(g, x) .. with b = rows / lanes, x = rows % lanes: the first x
 * lanes own b + 1 rows), a lane's codewords are cut into pieces of 8 (16 bytes, the last one
 * zero-padded), and the pieces of each group of 64 consecutive lanes are interleaved: piece p
 * of lane g is piece number wave_off[g / 64] + 64 p + g % 64 of the buffer, so that the 64
 * loads of a wavefront are 1 KiB of consecutive memory.  A group is as long as its longest
 * lane (shorter lanes are padded).  Same codewords, same order inside a lane; row_off keeps
 * its meaning (codeword counts), codes points to the pieces, n_codes is 8 * n_pieces.  The
 * padding is part of the compressed size: report 16 * n_pieces bytes, not 2 * row_off[rows].
 * Only the layer calls and qmoe_decompress read this layout, and only when their launch uses
 * exactly `lanes` lanes per matrix: pass the lane counts in the format argument
 * (QMOE_FORMAT_LANES) -- qmoe_plan_lanes gives the count the planner would pick.
 *   qmoe_lane_layout_size    number of 16-byte pieces the layout takes
 *   qmoe_lane_layout_build   codes (host, interchange or device numbering) -> out (host, 8 *
 *                            out_pieces codewords), wave_off (host [lanes/64 + 1])
 *   qmoe_lane_layout_unpack  the inverse (the layout round-trips)
 * lanes: a multiple of 64, 64 .. 16320.  Errors: INVALID_ARG, BUFFER_TOO_SMALL,
 * CORRUPT_STREAM (offsets that decrease), LIMIT (more than 2^32 - 1 pieces).
 */
qmoe_status qmoe_lane_layout_size(const uint32_t *row_off /*host [rows+1]*/, int rows, int lanes, size_t *n_pieces);
qmoe_status qmoe_lane_layout_build(const uint16_t *codes /*host*/, const uint32_t *row_off /*host [rows+1]*/, int rows,
                                   int lanes, uint16_t *out /*host*/, size_t out_pieces,
                                   uint32_t *wave_off /*host [lanes/64 + 1]*/);
qmoe_status qmoe_lane_layout_unpack(const uint16_t *pieces /*host*/, const uint32_t *wave_off /*host*/,
                                    const uint32_t *row_off /*host [rows+1]*/, int rows, int lanes,
                                    uint16_t *codes /*host*/, size_t codes_cap);
/*
 * Lanes per matrix that a layer call over n_experts experts and about n_tokens tokens would
 * use for a rows x cols projection of dictionary d (needs the GPU: the answer depends on its
 * LDS size); 0 on error.  Build the lane-interleaved layout of that projection for this count.
 */
int qmoe_plan_lanes(const qmoe_dict *d, int rows, int cols, int n_experts, int n_tokens);

/*
 * Format bits for the calls whose matrix descriptors live in device memory (the host
 * cannot look at them, so it is told): the `code_order` argument of qmoe_decompress,
 * qmoe_moe_layer_forward and qmoe_moe_dispatch is 0 or an OR of these.
 */
#define QMOE_FORMAT_DEVICE_ORDER 1 /* every stream uses the device numbering              */
#define QMOE_FORMAT_GRID_MINMAX 2  /* every matrix is on the asymmetric grid: the kernels
                                      read minmax_bf16 (a NULL there decodes to zeros)    */
/* every matrix is in the lane-interleaved layout, built for lanes_wi lanes (first product's
   matrices; the only ones of qmoe_decompress) and lanes_wo lanes (second product's); needs
   QMOE_FORMAT_DEVICE_ORDER */
#define QMOE_FORMAT_LANES(lanes_wi, lanes_wo) ((((lanes_wi) / 64) << 8) | (((lanes_wo) / 64) << 16))

/*
 * Rewrite a codeword stream in device memory, in place, from the interchange numbering
 * to the device numbering of d (see qmoe_dict_device_order): done once when a matrix is
 * loaded, like any weight pre-packing; the product kernels then find the whole table in
 * LDS.  Set code_order = 1 in the matrices that point into the rewritten stream.  Calling
 * it twice on the same codes garbles them.
 * Errors: INVALID_ARG, NO_DEVICE_DICT, LIMIT (the dictionary has no device order), HIP.
 */
qmoe_status qmoe_codes_to_device_order(const qmoe_dict *d, uint16_t *codes /*device*/, size_t n_codes,
                                       void *stream);

/*
 * Fused decode + product (the paper's kernel, extended by an inner loop over
 * tokens as its Section 5.3 suggests):
 *   y[b][r] = s_r * sum_c T[r][c] * x[b][c],  b < batch
 * (W->minmax_bf16 set: y[b][r] = w_max[r] * (sum of x under +1) + w_min[r] * (sum under -1))
 * W: host struct holding device pointers.  x: device bf16 [batch][cols].
 * y: device fp32 [batch][rows], overwritten.  fp32 accumulation.
 * One launch.  A small batch runs on a kernel that puts 16 lanes on every row (latency of a
 * single product); from a few dozen tokens on (device-order stream, cols divisible by 8, x
 * 16-byte aligned; the switch is a cost estimate, "mfma_min_tokens" overrides it) the matrix
 * is decoded once per 64 tokens and multiplied on the matrix cores.
 * Errors: INVALID_ARG (NULL, batch<1, odd cols), NO_DEVICE_DICT, LIMIT
 * (cols > 32768, or four tokens' activations, 8 bytes per column, do not fit the LDS: cols
 * above 20448 on a GPU with 160 KB), HIP.
 */
qmoe_status qmoe_decode_matvec(const qmoe_dict *d, const qmoe_matrix *W /*host*/,
                               const uint16_t *x_bf16 /*device*/, int batch, float *y /*device*/,
                               void *stream);

/*
 * Pure decompression (Section 4.3.3 mentions it as a variant): out is device
 * int8 [rows][cols] in {-1,0,+1} and equals the encoder's input bit for bit.
 * `path` selects the table the kernel reads: 0 = the one the product kernels
 * use for this dictionary, 1 = always the interchange layout.
 * Errors: as qmoe_decode_matvec.
 */
qmoe_status qmoe_decode_dense(const qmoe_dict *d, const qmoe_matrix *W /*host*/, int8_t *out /*device*/,
                              int path, void *stream);

/*
 * Decompress whole matrices (the codec of Section 4.3.3 without the product; the first
 * half of the alternative Section 5.3 names for experts with many tokens: decompress, then
 * multiply with a library routine):
 * out[m] receives matrix mats[m], row-major rows x cols, as int8 in {-1, 0, +1}
 * (out_kind 0) or as bf16 with the row scale folded in, bf16(s_r) * w (out_kind 1; with
 * QMOE_FORMAT_GRID_MINMAX the row's own w_min / w_max, which are bf16 already).
 * mats: device array [n_mats] of qmoe_matrix, all rows x cols, device numbering
 * (code_order must have QMOE_FORMAT_DEVICE_ORDER set).  out: device array [n_mats] of device pointers, 16-byte
 * aligned, NULL = skip that matrix.  cols must be a multiple of 8.  One launch for all
 * matrices; nothing is allocated.
 * Errors: INVALID_ARG, NO_DEVICE_DICT, LIMIT (no device order; cols > 32768; more matrices in
 * one call than the kernel's LDS has a bit for: about 20000 with the paper's table), HIP.
 */
qmoe_status qmoe_decompress(const qmoe_dict *d, const qmoe_matrix *mats /*device*/, int code_order,
                            int n_mats, int rows, int cols, int out_kind,
                            void *const *out /*device*/, void *stream);

/* ------------------------------------------------------------------------- */
/* One MoE feed-forward layer (Section 2.1; Section 5.1 on skipping experts)  */
/* ------------------------------------------------------------------------- */

/*
 * Where things live inside the layer workspace (byte offsets), for callers and
 * tests that want to look at the dispatch result:
 *   tok_off  int32 [n_experts+1]  expert e owns slots tok_off[e]..tok_off[e+1]
 *   perm     int32 [n_tokens]     slot -> token index, ascending inside an expert
 *   counters int32 [16]           [0] tokens kept, [1] tokens dropped (expert index
 *                                 outside [0,n_experts)), [2] experts with tokens,
 *                                 [3] work items of the first product, [4] of the second,
 *                                 [7] token tiles of crowded experts (items_mm, up to 64
 *                                 tokens each, both products, matrix-core kernel)
 *   items_*  int32 [n_tokens][4]  {expert, first slot, tokens, 0}; every kept token is in
 *                                 exactly one item of items_wi or items_mm, and one of
 *                                 items_wo or items_mm
 *   hidden   bf16  [n_tokens][d_ff]  by slot
 */
typedef struct qmoe_ws_layout {
    size_t tok_off, perm, counters, items_wi, items_wo, items_mm, hidden, total;
} qmoe_ws_layout;

qmoe_status qmoe_moe_layer_ws_layout(int n_experts, int d_model, int d_ff, int n_tokens,
                                     qmoe_ws_layout *out);
/* = layout.total; 0 on bad arguments */
size_t qmoe_moe_layer_workspace(int n_experts, int d_model, int d_ff, int n_tokens);

/*
 * y[t] = gate[t] * Wo[e] . bf16( relu( Wi[e] . x[t] ) ),  e = expert_idx[t]
 *
 * wi, wo: device arrays [n_experts] of qmoe_matrix (wi[e]: d_ff x d_model,
 * wo[e]: d_model x d_ff).  x: device bf16 [n_tokens][d_model].  expert_idx:
 * device int32 [n_tokens].  gate: device fp32 [n_tokens] or NULL (= 1).
 * y: device fp32 [n_tokens][d_model], overwritten; a token whose expert index
 * is outside [0, n_experts) gets a zero row.  workspace: device, 256-byte
 * aligned, >= qmoe_moe_layer_workspace(...) bytes, contents need not be
 * initialised.  Experts without tokens are never touched (their qmoe_matrix
 * may hold anything).  code_order: QMOE_FORMAT_* bits: the numbering of every expert's
 * stream (bit 0, as in qmoe_matrix) and whether the experts are on the asymmetric grid
 * (QMOE_FORMAT_GRID_MINMAX; the descriptors live in device memory, so the host is told).
 * Enqueues a dispatch kernel and, per product, the scalar kernel for experts with few
 * tokens and (device-order streams, widths divisible by 8, x 16-byte aligned) the
 * matrix-core kernel for crowded ones: an expert's matrix is decoded once per tile of up
 * to 64 tokens there, instead of once per 4.  When both kinds of experts are present the
 * two kernels of one kind run on a second stream that forks from `stream` after the dispatch and
 * joins it again before the call's work ends (two library-owned events per device), so that
 * later work on `stream` sees y complete as usual.  side_stream: that second stream, owned
 * by the caller like `stream` (default priority; it must not be `stream` itself); NULL = a
 * stream the library creates once per device and keeps.  Calls on one device must not be
 * issued concurrently from several host threads.
 * Errors: INVALID_ARG, NO_DEVICE_DICT, WORKSPACE, LIMIT (n_experts > 16384,
 * n_tokens > 2^20, d_model or d_ff > 32768, or too wide for the LDS: a token's activations
 * take 8 bytes per column, about 20400 columns with 160 KB (with the device numbering the
 * table shares the LDS with them up to 10022 columns and is read from L2, at about half the
 * speed, beyond that); code_order 1 without a device order), HIP.
 */
qmoe_status qmoe_moe_layer_forward(const qmoe_dict *d, const qmoe_matrix *wi /*device*/,
                                   const qmoe_matrix *wo /*device*/, int code_order, int n_experts,
                                   int d_model, int d_ff, const uint16_t *x_bf16 /*device*/,
                                   const int32_t *expert_idx /*device*/, const float *gate /*device*/,
                                   int n_tokens, float *y /*device*/, void *workspace /*device*/,
                                   size_t workspace_bytes, void *stream, void *side_stream);

/*
 * The same layer for callers that cannot allocate device memory or must not create
 * streams and events while they call: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  No workspace argument: the dispatch results, work
 * lists and the hidden vector live in a file-scope device array of
 * qmoe_static_workspace_bytes() = 8 MiB inside the library (each GPU the library runs on
 * holds its copy until the process ends).  All kernels are enqueued on `stream`, one after
 * the other (no second stream, no events); the call allocates nothing and creates nothing.
 * Limit: qmoe_moe_layer_workspace(n_experts, d_model, d_ff, n_tokens) must not exceed
 * qmoe_static_workspace_bytes(), else QMOE_E_LIMIT (e.g. 512 tokens at d_ff = 4096 fit,
 * 2048 tokens at d_ff = 6144 do not).  Every call on a GPU shares that GPU's array and
 * finds the previous call's contents there (the dispatch kernel rewrites all it reads);
 * calls that overlap on one GPU -- two streams, two host threads -- race.
 * Other arguments, results and errors as qmoe_moe_layer_forward.
 */
size_t qmoe_static_workspace_bytes(void);
qmoe_status qmoe_moe_layer_forward_static(const qmoe_dict *d, const qmoe_matrix *wi /*device*/,
                                          const qmoe_matrix *wo /*device*/, int code_order, int n_experts,
                                          int d_model, int d_ff, const uint16_t *x_bf16 /*device*/,
                                          const int32_t *expert_idx /*device*/, const float *gate /*device*/,
                                          int n_tokens, float *y /*device*/, void *stream);

/*
 * Only the dispatch step of the layer (fills tok_off, perm, counters, work items), planned
 * as qmoe_moe_layer_forward would for this dictionary and code order (and a 16-byte
 * aligned x).
 */
qmoe_status qmoe_moe_dispatch(const qmoe_dict *d, int code_order, const int32_t *expert_idx /*device*/,
                              int n_tokens, int n_experts, int d_model, int d_ff,
                              void *workspace /*device*/, size_t workspace_bytes, void *stream);

/*
 * The same layer on uncompressed bf16 weights, the execution the paper compares
 * against (Section 5.3): wi_dense[e] / wo_dense[e]
 * are device pointers to row-major bf16 matrices that already include the row
 * scales (NULL allowed for experts without tokens).  Same dispatch, same
 * workspace, same outputs.
 */
qmoe_status qmoe_bf16_layer_forward(const uint16_t *const *wi_dense /*device [n_experts]*/,
                                    const uint16_t *const *wo_dense /*device [n_experts]*/,
                                    int n_experts, int d_model, int d_ff,
                                    const uint16_t *x_bf16 /*device*/,
                                    const int32_t *expert_idx /*device*/, const float *gate /*device*/,
                                    int n_tokens, float *y /*device*/, void *workspace /*device*/,
                                    size_t workspace_bytes, void *stream);

/*
 * Launch tuning (process-wide, not thread-safe against running calls).  Keys:
 * "threads" (workgroup size of the scalar product kernel, a multiple of 64 up to 768),
 * "rows_per_item", "token_tile", "lds_dict_entries", "grid_per_cu",
 * "blocks_first" / "blocks_second" (workgroups that share one pass over a matrix in the
 * first or only / the second product), "mfma_min_tokens" (experts -- or, in
 * qmoe_decode_matvec, batches -- with at least this many tokens use the matrix-core kernel;
 * -1 = never), "overlap" (-1 = no side stream: all kernels of a layer one after the other on
 * the caller's stream), "host_threads" (encoder threads).  Value 0 restores the built-in
 * heuristic; lds_dict_entries = -1 keeps the whole table in L2 (either numbering), a
 * positive value forces it into LDS.
 * Unknown key: INVALID_ARG.
 */
qmoe_status qmoe_set_tuning(const char *key, int value);

/*
 * Plain device-to-device copy kernel (16 bytes per lane, grid-stride): the
 * yardstick for what a pure streaming kernel reaches on this GPU and the
 * calibration of the profiler's HBM byte counters.  dst, src: device, 16-byte
 * aligned, bytes a multiple of 16.  Errors: INVALID_ARG, HIP.
 */
qmoe_status qmoe_stream_copy(void *dst /*device*/, const void *src /*device*/, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QMOE_H */
