/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded reference for what the compressed-MoE hot
 * path computes: the static dictionary (Section 4.3.2, Algorithm 1), the
 * 64-bit entry layout (Section 4.3.2, "Dictionary Design and
 * Implementation"; bit positions as used by Listing 1), the longest-prefix
 * trie encoder (Section 4.3.3, "Encoding"), the sequential decoder
 * (Section 4.3.3, "Execution"), the dense ternary matrix-vector product in
 * fp64, and one MoE feed-forward block (Section 2.1).
 *
 * Nothing in the product path may call into this file: only the tests, the
 * smoke check and the benchmark's CPU-baseline leg do.  It shares no code
 * with the library or the HIP kernels.
 *
 * Every function here is pinned by tests that do not go through this file
 * (closed forms, brute force, numpy), see tests/test_oracle_*.py.
 *
 * Readings of the paper taken here:
 *  - a sequence holds 1..max_pairs pairs, max_pairs = 14 by default (the
 *    pair limit stated in the text of Section 4.3.2 above Algorithm 1, and the 2 x 7 slots
 *    of the entry format;
 *    Algorithm 1's strict "< 28" would leave the last slot unused);
 *  - the queue orders by probability, computed as a*ln(p0) + b*ln(q) from
 *    the integer counts a = #zeros, b = #non-zeros (q = (1-p0)/2), so that
 *    equal-probability sequences compare exactly equal; ties pop in
 *    ascending order of the symbol string read as a base-3 number;
 *  - symbols: 0 -> 0, 1 -> -s (the paper's w_min), 2 -> +s (w_max);
 *  - the asymmetric grid: 1 -> w_min[r], 2 -> w_max[r], one bfloat16 pair per
 *    output row as in the printed kernel's signature (Listing 1), no sign
 *    assumed for either; the symmetric case keeps its single binary16 scale;
 *  - entry word h (h = 0,1): bits 0..3 = total pair count, symbol j of the
 *    half at bits 4+2j, 4+2j+1 (14 symbols per word), unused slots 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define MAX_SYMS 28

/* ------------------------------------------------------------------ */
/* number formats                                                      */
/* ------------------------------------------------------------------ */

static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double f16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 31;
    int m = h & 1023;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

/* round a double to the nearest bfloat16 (ties to even), return its bits */
static uint16_t double_to_bf16(double d)
{
    /* The float nearest to d only serves to find d's two bfloat16 neighbours
       (the one at or below it in magnitude and the next one up); the choice
       between them is made on the double itself, so nothing is rounded twice. */
    float f = (float)d;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16);
    uint32_t lo = u & 0xFFFF0000u, hi = lo + 0x10000u;
    float flo, fhi;
    memcpy(&flo, &lo, 4);
    memcpy(&fhi, &hi, 4);
    double dl = fabs(d - (double)flo), dh = fabs((double)fhi - d);
    if (dl < dh) return (uint16_t)(lo >> 16);
    if (dh < dl) return (uint16_t)(hi >> 16);
    return (uint16_t)(((lo >> 16) & 1u) ? (hi >> 16) : (lo >> 16));
}

double orc_bf16_to_double(uint16_t b) { return bf16_to_double(b); }
double orc_f16_to_double(uint16_t h) { return f16_to_double(h); }
uint16_t orc_double_to_bf16(double d) { return double_to_bf16(d); }

/* ------------------------------------------------------------------ */
/* Algorithm 1: dictionary generation                                   */
/* ------------------------------------------------------------------ */

typedef struct {
    double logp;        /* a*ln(p0) + b*ln(q) */
    uint64_t base3;     /* symbol string as a base-3 number, first symbol most significant */
    int16_t zeros, nonzeros;
    uint8_t npairs;
    uint8_t sym[MAX_SYMS];
} seq_t;

/* 1 if x must pop before y */
static int pops_first(const seq_t *x, const seq_t *y)
{
    if (x->logp != y->logp) return x->logp > y->logp;
    return x->base3 < y->base3;
}

static void heap_push(seq_t *h, size_t *n, const seq_t *v)
{
    size_t i = (*n)++;
    h[i] = *v;
    while (i > 0) {
        size_t p = (i - 1) / 2;
        if (!pops_first(&h[i], &h[p])) break;
        seq_t t = h[i]; h[i] = h[p]; h[p] = t;
        i = p;
    }
}

static seq_t heap_pop(seq_t *h, size_t *n)
{
    seq_t top = h[0];
    h[0] = h[--(*n)];
    size_t i = 0;
    for (;;) {
        size_t l = 2 * i + 1, r = l + 1, m = i;
        if (l < *n && pops_first(&h[l], &h[m])) m = l;
        if (r < *n && pops_first(&h[r], &h[m])) m = r;
        if (m == i) break;
        seq_t t = h[i]; h[i] = h[m]; h[m] = t;
        i = m;
    }
    return top;
}

/*
 * Build the dictionary.  syms: [n_entries][28] (unused slots 0),
 * npairs: [n_entries].  Returns the number of entries produced (fewer than
 * n_entries only when fewer sequences exist), or -1 on bad arguments.
 *
 * Follows Algorithm 1: start from the empty sequence, pop the most probable
 * sequence, append it if it holds 1..max_pairs pairs, push its nine one-pair
 * extensions.  Extensions of a sequence that already holds max_pairs pairs
 * are not pushed: neither they nor anything grown from them could ever be
 * appended, so the dictionary is the same and the queue stays bounded.
 */
int orc_dict_build(double p0, int max_pairs, int n_entries, uint8_t *syms, uint8_t *npairs)
{
    if (!(p0 > 0.0 && p0 < 1.0) || max_pairs < 1 || max_pairs > 14 || n_entries < 1) return -1;
    const double lp0 = log(p0), lq = log((1.0 - p0) / 2.0);
    size_t cap = (size_t)9 * (size_t)(n_entries + 2) + 16, n = 0;
    seq_t *heap = (seq_t *)malloc(cap * sizeof(seq_t));
    if (!heap) return -1;
    seq_t root;
    memset(&root, 0, sizeof root);
    heap_push(heap, &n, &root);
    int count = 0;
    while (count < n_entries && n > 0) {
        seq_t s = heap_pop(heap, &n);
        if (s.npairs >= 1 && s.npairs <= max_pairs) {
            memcpy(syms + (size_t)count * MAX_SYMS, s.sym, MAX_SYMS);
            npairs[count] = s.npairs;
            count++;
        }
        if (s.npairs >= max_pairs) continue;
        for (int t1 = 0; t1 < 3; t1++)
            for (int t2 = 0; t2 < 3; t2++) {
                seq_t c = s;
                c.sym[2 * s.npairs] = (uint8_t)t1;
                c.sym[2 * s.npairs + 1] = (uint8_t)t2;
                c.npairs = (uint8_t)(s.npairs + 1);
                c.zeros = (int16_t)(s.zeros + (t1 == 0) + (t2 == 0));
                c.nonzeros = (int16_t)(s.nonzeros + (t1 != 0) + (t2 != 0));
                c.base3 = (s.base3 * 3u + (uint64_t)t1) * 3u + (uint64_t)t2;
                c.logp = (double)c.zeros * lp0 + (double)c.nonzeros * lq;
                if (n < cap) heap_push(heap, &n, &c);
            }
    }
    free(heap);
    return count;
}

/* 64-bit entry layout: two 32-bit words, 7 pairs each, count in both low nibbles */
void orc_dict_pack(const uint8_t *syms, const uint8_t *npairs, int n, uint32_t *words)
{
    for (int k = 0; k < n; k++)
        for (int h = 0; h < 2; h++) {
            uint32_t w = npairs[k] & 15u;
            for (int j = 0; j < 14; j++)
                w |= (uint32_t)(syms[(size_t)k * MAX_SYMS + 14 * h + j] & 3u) << (4 + 2 * j);
            words[2 * (size_t)k + h] = w;
        }
}

/* ------------------------------------------------------------------ */
/* Encoder: trie over the dictionary, longest prefix match              */
/* ------------------------------------------------------------------ */

typedef struct { int32_t child[9]; int32_t code; } tnode;

typedef struct { tnode *nodes; int n_nodes; } trie_t;

static int trie_build(trie_t *t, const uint8_t *syms, const uint8_t *npairs, int n)
{
    size_t cap = (size_t)n * 14 + 1;
    t->nodes = (tnode *)malloc(cap * sizeof(tnode));
    if (!t->nodes) return -1;
    t->n_nodes = 1;
    memset(t->nodes[0].child, 0xFF, sizeof t->nodes[0].child);
    t->nodes[0].code = -1;
    for (int k = 0; k < n; k++) {
        int cur = 0;
        for (int j = 0; j < npairs[k]; j++) {
            int pr = 3 * syms[(size_t)k * MAX_SYMS + 2 * j] + syms[(size_t)k * MAX_SYMS + 2 * j + 1];
            if (t->nodes[cur].child[pr] < 0) {
                int nn = t->n_nodes++;
                memset(t->nodes[nn].child, 0xFF, sizeof t->nodes[nn].child);
                t->nodes[nn].code = -1;
                t->nodes[cur].child[pr] = nn;
            }
            cur = t->nodes[cur].child[pr];
        }
        if (t->nodes[cur].code < 0) t->nodes[cur].code = k; /* first (most probable) wins */
    }
    return 0;
}

static int sym_of(int8_t v) { return v == 0 ? 0 : (v < 0 ? 1 : 2); }

/*
 * Encode a row-major ternary matrix (int8 in {-1,0,+1}).  Each row is an
 * independent stream; rows are packed back to back and row_off[r] is the
 * index of row r's first codeword (row_off[rows] = total).  codes may be
 * NULL to only count.  Returns 0, or 1 bad symbol, 2 odd cols, 3 capacity,
 * 4 a phrase that no dictionary entry starts, -1 out of memory.
 */
int orc_encode(const uint8_t *syms, const uint8_t *npairs, int n_entries, const int8_t *tern,
               int64_t rows, int64_t cols, uint16_t *codes, uint64_t codes_cap, uint32_t *row_off,
               uint64_t *n_codes)
{
    if (cols % 2) return 2;
    trie_t t;
    if (trie_build(&t, syms, npairs, n_entries)) return -1;
    uint64_t out = 0;
    int rc = 0;
    int64_t np = cols / 2;
    for (int64_t r = 0; r < rows && !rc; r++) {
        const int8_t *row = tern + r * cols;
        row_off[r] = (uint32_t)out;
        int64_t i = 0;
        while (i < np) {
            int cur = 0, best = -1;
            int64_t best_len = 0, d = 0;
            while (i + d < np) {
                int8_t a = row[2 * (i + d)], b = row[2 * (i + d) + 1];
                if (a < -1 || a > 1 || b < -1 || b > 1) { rc = 1; break; }
                int nx = t.nodes[cur].child[3 * sym_of(a) + sym_of(b)];
                if (nx < 0) break;
                cur = nx;
                d++;
                if (t.nodes[cur].code >= 0) { best = t.nodes[cur].code; best_len = d; }
            }
            if (rc) break;
            if (best < 0) { rc = 4; break; }
            if (codes) {
                if (out >= codes_cap) { rc = 3; break; }
                codes[out] = (uint16_t)best;
            }
            out++;
            i += best_len;
        }
    }
    row_off[rows] = (uint32_t)out;
    *n_codes = out;
    free(t.nodes);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Decoder                                                              */
/* ------------------------------------------------------------------ */

/*
 * Decode from the packed entry words.  Walks each row's codewords in order,
 * writing 2*npairs symbols per codeword at a running column index that must
 * end exactly at cols.  Returns 0, or 1 row over/under-run, 2 codeword out
 * of range, 3 symbol value 3, 4 the two count nibbles differ.
 */
int orc_decode(const uint32_t *words, int n_entries, const uint16_t *codes, const uint32_t *row_off,
               int64_t rows, int64_t cols, int8_t *out)
{
    for (int64_t r = 0; r < rows; r++) {
        int64_t idx = 0;
        for (uint32_t k = row_off[r]; k < row_off[r + 1]; k++) {
            uint32_t c = codes[k];
            if ((int)c >= n_entries) return 2;
            uint32_t w0 = words[2 * c], w1 = words[2 * c + 1];
            int np = (int)(w0 & 15u);
            if ((int)(w1 & 15u) != np) return 4;
            if (idx + 2 * np > cols) return 1;
            for (int j = 0; j < 2 * np; j++) {
                uint32_t w = j < 14 ? w0 : w1;
                int s = (int)((w >> (4 + 2 * (j % 14))) & 3u);
                if (s == 3) return 3;
                out[r * cols + idx + j] = (int8_t)(s == 0 ? 0 : (s == 1 ? -1 : 1));
            }
            idx += 2 * np;
        }
        if (idx != cols) return 1;
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Dense ternary matrix-vector product, fp64                            */
/* ------------------------------------------------------------------ */

/*
 * y[b][r] = sum_c value_r(T[r][c]) * x[b][c], value_r(+1) = w_max[r], value_r(-1) = w_min[r],
 * value_r(0) = 0: the per-row grid {w_min, 0, w_max} of Section 4.1 (symbols 0, 1, 2
 * dequantise to 0, w_min, w_max: "Ternary decoding", Section 4.3.3).
 * T int8 {-1,0,+1} [rows][cols]; minmax bfloat16 bits [rows][2] = (w_min, w_max) of each
 * row, of any sign; x bfloat16 bits [batch][cols]; y double [batch][rows].  The inputs
 * under w_max and those under w_min are summed apart and each sum is scaled once.  Also
 * returns, when abs_sum is not NULL, sum_c |value_r(T[r][c]) * x[b][c]| (the scale of the
 * rounding-error bound used by the parity tests).
 */
void orc_matvec_asym(const int8_t *tern, const uint16_t *minmax_bf16, const uint16_t *x_bf16, int64_t rows,
                     int64_t cols, int64_t batch, double *y, double *abs_sum)
{
    for (int64_t b = 0; b < batch; b++)
        for (int64_t r = 0; r < rows; r++) {
            double hi = 0.0, lo = 0.0, hi_mag = 0.0, lo_mag = 0.0;
            for (int64_t c = 0; c < cols; c++) {
                double xv = bf16_to_double(x_bf16[b * cols + c]);
                if (tern[r * cols + c] > 0) {
                    hi += xv;
                    hi_mag += fabs(xv);
                } else if (tern[r * cols + c] < 0) {
                    lo += xv;
                    lo_mag += fabs(xv);
                }
            }
            double w_min = bf16_to_double(minmax_bf16[2 * r]), w_max = bf16_to_double(minmax_bf16[2 * r + 1]);
            y[b * rows + r] = w_max * hi + w_min * lo;
            if (abs_sum) abs_sum[b * rows + r] = fabs(w_max) * hi_mag + fabs(w_min) * lo_mag;
        }
}

/*
 * y[b][r] = s_r * sum_c T[r][c] * x[b][c]: the symmetric grid {-s, 0, +s}, written out
 * on its own (one signed sum, scaled once).
 */
void orc_matvec(const int8_t *tern, const uint16_t *scale_f16, const uint16_t *x_bf16, int64_t rows,
                int64_t cols, int64_t batch, double *y, double *abs_sum)
{
    for (int64_t b = 0; b < batch; b++)
        for (int64_t r = 0; r < rows; r++) {
            double acc = 0.0, mag = 0.0;
            for (int64_t c = 0; c < cols; c++) {
                double term = (double)tern[r * cols + c] * bf16_to_double(x_bf16[b * cols + c]);
                acc += term;
                mag += fabs(term);
            }
            double s = f16_to_double(scale_f16[r]);
            y[b * rows + r] = s * acc;
            if (abs_sum) abs_sum[b * rows + r] = fabs(s) * mag;
        }
}

/*
 * One token through one expert's feed-forward block (Section 2.1):
 *   h = bf16( relu( Wi x ) ),  y = gate * Wo h
 * Wi [d_ff][d_model], Wo [d_model][d_ff]; h_bf16 (optional) receives the
 * rounded hidden vector; abs_sum (optional) the error-bound scale of the
 * second product, gate * s_r * sum |Wo h|.
 */
void orc_ffn_token_asym(const int8_t *wi, const uint16_t *wi_scale, const uint16_t *wi_minmax, const int8_t *wo,
                        const uint16_t *wo_scale, const uint16_t *wo_minmax, const uint16_t *x_bf16,
                        int64_t d_model, int64_t d_ff, double gate, double *y, uint16_t *h_bf16, double *abs_sum)
{
    double *h = (double *)malloc((size_t)d_ff * sizeof(double));
    uint16_t *hb = (uint16_t *)malloc((size_t)d_ff * sizeof(uint16_t));
    if (wi_minmax)
        orc_matvec_asym(wi, wi_minmax, x_bf16, d_ff, d_model, 1, h, NULL);
    else
        orc_matvec(wi, wi_scale, x_bf16, d_ff, d_model, 1, h, NULL);
    for (int64_t i = 0; i < d_ff; i++) {
        double v = h[i] > 0.0 ? h[i] : 0.0;
        hb[i] = double_to_bf16(v);
    }
    if (wo_minmax)
        orc_matvec_asym(wo, wo_minmax, hb, d_model, d_ff, 1, y, abs_sum);
    else
        orc_matvec(wo, wo_scale, hb, d_model, d_ff, 1, y, abs_sum);
    for (int64_t i = 0; i < d_model; i++) {
        y[i] *= gate;
        if (abs_sum) abs_sum[i] *= fabs(gate);
    }
    if (h_bf16) memcpy(h_bf16, hb, (size_t)d_ff * sizeof(uint16_t));
    free(h);
    free(hb);
}

void orc_ffn_token(const int8_t *wi, const uint16_t *wi_scale, const int8_t *wo,
                   const uint16_t *wo_scale, const uint16_t *x_bf16, int64_t d_model, int64_t d_ff,
                   double gate, double *y, uint16_t *h_bf16, double *abs_sum)
{
    orc_ffn_token_asym(wi, wi_scale, NULL, wo, wo_scale, NULL, x_bf16, d_model, d_ff, gate, y, h_bf16, abs_sum);
}

/* ------------------------------------------------------------------ */
/* Second formulation of the product: the slot-parallel decoder          */
/* ------------------------------------------------------------------ */

/*
 * The product as the paper's kernel computes it (Section 4.3.3, "Execution" and
 * Listing 1), straight from the packed entry words and the codeword stream, without
 * ever materialising the matrix: 28 workers, one per slot of a dictionary entry.  For
 * every codeword of a row, worker j reads symbol j of the entry (slot j of the first
 * word for j < 14, slot j - 14 of the second otherwise), dequantises it through the
 * row's three-value table {0, w_min, w_max} and adds value * x[start + j] to its own
 * partial sum; `start` then advances by twice the entry's pair count.  Nothing tests j
 * against the entry's length: slots past it hold symbol 0, and x is read up to 27
 * places past the row's end, where it is zero-padded.  The 28 partial sums are added at
 * the end of the row.  fp64 throughout; result overwrites y (the printed kernel adds
 * into a bfloat16 y).
 * minmax: [rows][2] doubles (w_min, w_max) of each row.  Returns 0, or 2 for a codeword
 * outside the table, 1 for a row whose phrases run past cols + 28.
 */
int orc_slot_parallel_matvec(const uint32_t *words, int n_entries, const uint16_t *codes, const uint32_t *row_off,
                             const double *minmax, const uint16_t *x_bf16, int64_t rows, int64_t cols, double *y)
{
    enum { SLOTS = 28 };
    double *xpad = (double *)calloc((size_t)cols + SLOTS, sizeof(double));
    if (!xpad) return -1;
    for (int64_t c = 0; c < cols; c++) xpad[c] = bf16_to_double(x_bf16[c]);
    int rc = 0;
    for (int64_t r = 0; r < rows && !rc; r++) {
        const double deq[3] = {0.0, minmax[2 * r], minmax[2 * r + 1]};
        double part[SLOTS];
        for (int j = 0; j < SLOTS; j++) part[j] = 0.0;
        int64_t start = 0;
        for (uint32_t k = row_off[r]; k < row_off[r + 1]; k++) {
            const uint32_t enc = codes[k];
            if ((int)enc >= n_entries) { rc = 2; break; }
            if (start > cols) { rc = 1; break; }
            const uint32_t *w = words + 2 * (size_t)enc;
            for (int j = 0; j < SLOTS; j++) {
                const uint32_t half = w[j / 14];
                const unsigned sym = (half >> (4 + 2 * (j % 14))) & 3u;
                if (sym == 3u) { rc = 3; break; }
                part[j] += deq[sym] * xpad[start + j];
            }
            start += 2 * (int64_t)(w[0] & 15u);
        }
        double sum = 0.0;
        for (int j = 0; j < SLOTS; j++) sum += part[j];
        y[r] = sum;
    }
    free(xpad);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Token dispatch: group tokens by expert, keeping their order          */
/* ------------------------------------------------------------------ */

/*
 * tok_off[e]..tok_off[e+1] is expert e's slice of perm; perm lists token
 * indices, ascending within each expert.  Tokens whose index is outside
 * [0, n_experts) are left out (tok_off[n_experts] counts the rest).
 */
void orc_dispatch(const int32_t *expert_idx, int64_t n_tokens, int64_t n_experts, int32_t *tok_off,
                  int32_t *perm)
{
    for (int64_t e = 0; e <= n_experts; e++) tok_off[e] = 0;
    for (int64_t t = 0; t < n_tokens; t++)
        if (expert_idx[t] >= 0 && expert_idx[t] < n_experts) tok_off[expert_idx[t] + 1]++;
    for (int64_t e = 0; e < n_experts; e++) tok_off[e + 1] += tok_off[e];
    int32_t *cur = (int32_t *)malloc((size_t)(n_experts + 1) * sizeof(int32_t));
    memcpy(cur, tok_off, (size_t)(n_experts + 1) * sizeof(int32_t));
    for (int64_t t = 0; t < n_tokens; t++)
        if (expert_idx[t] >= 0 && expert_idx[t] < n_experts) perm[cur[expert_idx[t]]++] = (int32_t)t;
    free(cur);
}
