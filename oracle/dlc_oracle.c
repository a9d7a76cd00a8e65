/*
 * dlc_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, single-threaded CPU statement of the error-bounded embedding
 * payload compressor of "Accelerating Communication in DLRM Training with
 * Dual-Level Adaptive Lossy Compression" (arXiv 2407.04272): quantisation
 * encoder without prediction followed by a Huffman entropy encoder
 * (Section III-D), driven by the table-wise / iteration-wise error-bound
 * strategy of Section III-C (Eq. 1, Algorithm 1).
 *
 * Only tests, the smoke check and the bench's CPU-baseline leg may use it.
 * It shares no code, header, table or helper with the HIP library; the
 * product path never calls into this file.
 *
 * The paper fixes the structure of the method and nothing about number
 * formats, tie-breaks or byte layout.  Every such choice made here is a
 * "reading" and is listed next to the function that takes it.
 *
 * Pins (see tests/test_oracle_*.py): Homo-Index values printed in Tables
 * III and IV; the 0.05/0.03/0.01 class bounds of Section IV-B; the point-wise
 * bound on every element; exact-rational rounding; numpy fp16 conversion;
 * numpy.bincount; prefix property, Kraft equality, optimal cost against an
 * independent heap Huffman and brute force; an independent Python stream
 * reader.  Unpinned (no value in the paper to check against): the class
 * thresholds and the placement of the staircase steps ("parity unpinned").
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ENOMEM (-2)
#define ORC_ECAPACITY (-3)
#define ORC_ECORRUPT (-4)

#define ORC_F32 0
#define ORC_F16 1

/* container constants (a reading: the paper gives no layout) */
#define ORC_MAGIC 0x32434C44u /* "DLC2" */
#define ORC_VERSION 2u
#define ORC_W 64u /* chunks per group */
#define ORC_V 4u  /* consecutive symbols a chunk takes per turn */
#define ORC_HEADER_BYTES 128u
#define ORC_DIR_BYTES 56u
#define ORC_LMAX_LIMIT 12

/* ------------------------------------------------------------------ */
/* half precision <-> single precision, written out bit by bit         */
/* ------------------------------------------------------------------ */

/* IEEE binary16 -> binary32, exact. */
float orc_half_to_float(uint16_t h) {
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t e = (h >> 10) & 0x1Fu;
    uint32_t m = h & 0x3FFu;
    uint32_t bits;
    if (e == 0) {
        if (m == 0) {
            bits = sign;
        } else { /* subnormal half: value = m * 2^-24 */
            float v = (float)m * 5.9604644775390625e-08f; /* exact product */
            memcpy(&bits, &v, 4);
            bits |= sign;
        }
    } else if (e == 31) {
        bits = sign | 0x7F800000u | (m << 13);
    } else {
        bits = sign | ((e + 112u) << 23) | (m << 13);
    }
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

/* IEEE binary32 -> binary16, round to nearest, ties to even. */
uint16_t orc_float_to_half(float f) {
    uint32_t x;
    memcpy(&x, &f, 4);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t a = x & 0x7FFFFFFFu;
    if (a >= 0x7F800000u) { /* inf or nan */
        if (a == 0x7F800000u) return (uint16_t)(sign | 0x7C00u);
        uint16_t m = (uint16_t)((a >> 13) & 0x3FFu);
        return (uint16_t)(sign | 0x7C00u | m | 0x200u); /* quiet */
    }
    if (a >= 0x477FF000u) { /* >= 65520 rounds to infinity */
        return (uint16_t)(sign | 0x7C00u);
    }
    if (a < 0x33000001u) { /* <= 2^-25: rounds to zero (tie at 2^-25 goes to even = 0) */
        return sign;
    }
    int32_t e = (int32_t)(a >> 23) - 127;
    uint32_t m = (a & 0x7FFFFFu) | 0x800000u; /* 24-bit significand */
    uint32_t shift;                           /* bits to drop */
    uint32_t base;
    if (e >= -14) {
        shift = 13;
        base = (uint32_t)(e + 15) << 10;
        m &= 0x7FFFFFu; /* hidden bit is carried by the exponent field */
    } else {
        shift = (uint32_t)(13 + (-14 - e)); /* subnormal half */
        base = 0;
    }
    uint32_t q = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t halfway = 1u << (shift - 1);
    if (rem > halfway || (rem == halfway && (q & 1u))) q += 1; /* may carry into exponent: intended */
    return (uint16_t)(sign | (base + q));
}

/* ------------------------------------------------------------------ */
/* Quantisation encoder, Section III-D; no predictor (observation 1).  */
/*                                                                     */
/* Reading: bins of width 2*eb centred on multiples of 2*eb; the code  */
/* of an element is its bin number plus R.  An element whose bin lies  */
/* outside (-R, R), or whose reconstruction would miss the point-wise  */
/* bound of Section III-C, takes the escape symbol 0 and is kept       */
/* verbatim.  All arithmetic is IEEE binary32, one operation at a time.*/
/* ------------------------------------------------------------------ */

typedef struct {
    float eb;
    float ebx2;
    float inv;
} orc_qparam;

static orc_qparam make_qparam(float eb) {
    orc_qparam q;
    q.eb = eb;
    q.ebx2 = eb * 2.0f;
    q.inv = (float)(1.0 / (double)q.ebx2);
    return q;
}

static float load_elem(const void* p, int dtype, size_t i) {
    if (dtype == ORC_F16) return orc_half_to_float(((const uint16_t*)p)[i]);
    return ((const float*)p)[i];
}

static uint32_t load_raw(const void* p, int dtype, size_t i) {
    if (dtype == ORC_F16) return ((const uint16_t*)p)[i];
    return ((const uint32_t*)p)[i];
}

/* symbol of one element; *recon gets the value a decoder would produce
 * for a non-escape symbol (unspecified for escapes). */
static uint32_t quantize_one(float x, const orc_qparam* q, int dtype, int R, float* recon) {
    volatile float prod = x * q->inv;
    float r = rintf(prod); /* default rounding mode: nearest, ties to even */
    int in_range = fabsf(r) < (float)R;
    volatile float xh = r * q->ebx2;
    float xhat = xh;
    if (dtype == ORC_F16) xhat = orc_half_to_float(orc_float_to_half(xhat));
    volatile float diff = x - xhat;
    int ok = in_range && (fabsf(diff) <= q->eb);
    *recon = xhat;
    if (!ok) return 0;
    return (uint32_t)((int)r + R);
}

/* value a decoder produces for symbol c (c != 0) at bound eb */
static float dequantize_one(uint32_t c, const orc_qparam* q, int R) {
    volatile float v = (float)((int)c - R) * q->ebx2;
    return v;
}

/* symbols (u16) of n elements at one bound; optional reconstruction
 * (same dtype as the input: escapes reconstruct to the input itself). */
int orc_quantize(const void* x, int dtype, size_t n, float eb, int R, uint16_t* sym, void* recon) {
    if (!x || !sym || !(eb > 0.0f) || isinf(eb) || R < 2 || R > 2048) return ORC_EINVAL;
    orc_qparam q = make_qparam(eb);
    for (size_t i = 0; i < n; ++i) {
        float xi = load_elem(x, dtype, i);
        float xh;
        uint32_t c = quantize_one(xi, &q, dtype, R, &xh);
        sym[i] = (uint16_t)c;
        if (recon) { /* what the decoder produces: (c - R) * 2eb, so bin 0 is +0.0 whatever the sign of x */
            if (c) xh = dequantize_one(c, &q, R);
            if (dtype == ORC_F16) {
                ((uint16_t*)recon)[i] = c ? orc_float_to_half(xh) : ((const uint16_t*)x)[i];
            } else {
                if (c) ((float*)recon)[i] = xh;
                else ((uint32_t*)recon)[i] = ((const uint32_t*)x)[i];
            }
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* Code histogram (implied by the entropy encoder of Section III-D).   */
/* ------------------------------------------------------------------ */
int orc_histogram(const uint16_t* sym, size_t n, int K, uint64_t* hist) {
    if (!sym || !hist || K < 1) return ORC_EINVAL;
    for (int k = 0; k < K; ++k) hist[k] = 0;
    for (size_t i = 0; i < n; ++i) {
        if (sym[i] >= K) return ORC_EINVAL;
        hist[sym[i]] += 1;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* Huffman code lengths and canonical codewords (Section III-D names   */
/* Huffman; every tie-break below is a reading).                       */
/*                                                                     */
/*  - leaves ordered by (count, symbol) ascending                      */
/*  - two queues: sorted leaves, and merged nodes in creation order;   */
/*    each pick takes the smaller head, a tie goes to the leaf queue   */
/*  - if the longest code exceeds LMAX: lengths above LMAX are cut to  */
/*    LMAX; while the Kraft sum is too large, one code of length LMAX  */
/*    is paired with a code taken from the deepest shorter level (that */
/*    level loses one code, the next gains two), which lowers the sum  */
/*    by one unit of 2^-LMAX; the resulting number of codes per length */
/*    is handed out most frequent symbol first (the classic length     */
/*    adjustment of JPEG Annex K / deflate encoders)                   */
/*  - one used symbol: length 0                                        */
/*  - codewords: symbols ordered by (length, symbol); first code 0;    */
/*    next = (previous + 1) << (length increase)                       */
/* ------------------------------------------------------------------ */
typedef struct {
    uint64_t count;
    uint32_t sym;
} orc_leaf;

static int leaf_cmp(const void* a, const void* b) {
    const orc_leaf* x = (const orc_leaf*)a;
    const orc_leaf* y = (const orc_leaf*)b;
    if (x->count != y->count) return x->count < y->count ? -1 : 1;
    if (x->sym != y->sym) return x->sym < y->sym ? -1 : 1;
    return 0;
}

/* lengths of the leaves (in leaf order) of the Huffman tree over n >= 2
 * sorted leaves; returns the longest */
static int huffman_depths(const orc_leaf* leaf, int n, int* depth) {
    int n_int = n - 1;
    uint64_t* w = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)n_int);
    int* parent_leaf = (int*)malloc(sizeof(int) * (size_t)n);
    int* parent_int = (int*)malloc(sizeof(int) * (size_t)n_int);
    int* d_int = (int*)malloc(sizeof(int) * (size_t)n_int);
    int a = 0; /* head of leaf queue */
    int b = 0; /* head of merged-node queue */
    for (int k = 0; k < n_int; ++k) {
        uint64_t sum = 0;
        for (int pick = 0; pick < 2; ++pick) {
            int take_leaf;
            if (a >= n) take_leaf = 0;
            else if (b >= k) take_leaf = 1;
            else take_leaf = leaf[a].count <= w[b];
            if (take_leaf) {
                sum += leaf[a].count;
                parent_leaf[a] = k;
                a++;
            } else {
                sum += w[b];
                parent_int[b] = k;
                b++;
            }
        }
        w[k] = sum;
    }
    d_int[n_int - 1] = 0; /* root */
    for (int k = n_int - 2; k >= 0; --k) d_int[k] = d_int[parent_int[k]] + 1;
    int longest = 0;
    for (int i = 0; i < n; ++i) {
        depth[i] = d_int[parent_leaf[i]] + 1;
        if (depth[i] > longest) longest = depth[i];
    }
    free(w);
    free(parent_leaf);
    free(parent_int);
    free(d_int);
    return longest;
}

int orc_codebook(const uint64_t* hist, int K, int LMAX, uint8_t* len, uint32_t* code, int* n_used_out,
                 int* n_repairs_out) {
    if (!hist || !len || !code || K < 2 || K > 4096 || LMAX < 1 || LMAX > ORC_LMAX_LIMIT) return ORC_EINVAL;
    if ((1 << LMAX) < K) return ORC_EINVAL; /* a code for every symbol must exist */
    orc_leaf* leaf = (orc_leaf*)malloc(sizeof(orc_leaf) * (size_t)K);
    int* depth = (int*)malloc(sizeof(int) * (size_t)K);
    int n = 0;
    for (int k = 0; k < K; ++k) {
        len[k] = 0;
        code[k] = 0;
        if (hist[k]) {
            leaf[n].count = hist[k];
            leaf[n].sym = (uint32_t)k;
            n++;
        }
    }
    int repairs = 0; /* number of Kraft repair steps (0: plain Huffman) */
    if (n >= 2) {
        qsort(leaf, (size_t)n, sizeof(orc_leaf), leaf_cmp);
        int longest = huffman_depths(leaf, n, depth);
        if (longest > LMAX) {
            uint32_t per_len[ORC_LMAX_LIMIT + 2];
            memset(per_len, 0, sizeof per_len);
            for (int i = 0; i < n; ++i) per_len[depth[i] > LMAX ? LMAX : depth[i]] += 1;
            uint64_t kraft = 0;
            for (int L = 1; L <= LMAX; ++L) kraft += (uint64_t)per_len[L] << (LMAX - L);
            while (kraft > (1ull << LMAX)) {
                per_len[LMAX] -= 1;
                for (int L = LMAX - 1; L >= 1; --L)
                    if (per_len[L]) {
                        per_len[L] -= 1;
                        per_len[L + 1] += 2;
                        break;
                    }
                kraft -= 1;
                repairs++;
            }
            int i = n - 1; /* leaves are sorted by rising count: the last one is the most frequent */
            for (int L = 1; L <= LMAX; ++L)
                for (uint32_t c = 0; c < per_len[L]; ++c) depth[i--] = L;
        }
        for (int i = 0; i < n; ++i) len[leaf[i].sym] = (uint8_t)depth[i];
        /* canonical codewords in (length, symbol) order */
        uint32_t next = 0;
        int prev_len = 0;
        int first = 1;
        for (int L = 1; L <= LMAX; ++L) {
            for (int k = 0; k < K; ++k) {
                if (len[k] != L) continue;
                if (first) {
                    next = 0;
                    first = 0;
                } else {
                    next = (next + 1) << (L - prev_len);
                }
                prev_len = L;
                code[k] = next;
            }
        }
    }
    if (n_used_out) *n_used_out = n;
    if (n_repairs_out) *n_repairs_out = repairs;
    free(leaf);
    free(depth);
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* Per-table statistics and the Homogenization Index, Eq. 1:           */
/*   eta = (N_original - N_compressed) / N_original                    */
/* N_original  = distinct rows of the sampled batch (raw bit patterns) */
/* N_compressed = distinct rows after quantisation at a probe bound    */
/* Reading: Tables III/IV print N_quant/N_ori, which is 1 - eta.       */
/* ------------------------------------------------------------------ */
typedef struct {
    float min;              /* over finite elements; +inf if none */
    float max;              /* over finite elements; -inf if none */
    uint64_t count;         /* elements in the table's batch */
    uint32_t n_rows;        /* B */
    uint32_t n_unique_raw;  /* N_original */
    uint32_t n_unique_quant;/* N_compressed */
    float probe_eb;
} orc_table_stats;

static size_t g_row_bytes;
static int row_cmp(const void* a, const void* b) {
    return memcmp(*(const void* const*)a, *(const void* const*)b, g_row_bytes);
}

static uint32_t count_distinct_rows(const uint8_t* base, size_t n_rows, size_t row_bytes) {
    const void** ptr = (const void**)malloc(sizeof(void*) * n_rows);
    for (size_t i = 0; i < n_rows; ++i) ptr[i] = base + i * row_bytes;
    g_row_bytes = row_bytes;
    qsort(ptr, n_rows, sizeof(void*), row_cmp);
    uint32_t distinct = n_rows ? 1u : 0u;
    for (size_t i = 1; i < n_rows; ++i)
        if (memcmp(ptr[i - 1], ptr[i], row_bytes) != 0) distinct++;
    free(ptr);
    return distinct;
}

int orc_stats(const void* payload, int dtype, int T, int64_t B, int64_t D, int R, const float* probe_eb,
              orc_table_stats* out) {
    if (!payload || !probe_eb || !out || T < 1 || B < 1 || D < 1) return ORC_EINVAL;
    size_t es = dtype == ORC_F16 ? 2 : 4;
    size_t n = (size_t)B * (size_t)D;
    uint16_t* sym = (uint16_t*)malloc(sizeof(uint16_t) * n);
    if (!sym) return ORC_ENOMEM;
    for (int t = 0; t < T; ++t) {
        const uint8_t* tab = (const uint8_t*)payload + (size_t)t * n * es;
        float mn = INFINITY, mx = -INFINITY;
        for (size_t i = 0; i < n; ++i) {
            float x = load_elem(tab, dtype, i);
            if (isfinite(x)) {
                if (x < mn) mn = x;
                if (x > mx) mx = x;
            }
        }
        int rc = orc_quantize(tab, dtype, n, probe_eb[t], R, sym, NULL);
        if (rc != ORC_OK) {
            free(sym);
            return rc;
        }
        out[t].min = mn;
        out[t].max = mx;
        out[t].count = n;
        out[t].n_rows = (uint32_t)B;
        out[t].n_unique_raw = count_distinct_rows(tab, (size_t)B, (size_t)D * es);
        out[t].n_unique_quant = count_distinct_rows((const uint8_t*)sym, (size_t)B, (size_t)D * 2);
        out[t].probe_eb = probe_eb[t];
    }
    free(sym);
    return ORC_OK;
}

double orc_homo_index(uint32_t n_original, uint32_t n_compressed) {
    return ((double)n_original - (double)n_compressed) / (double)n_original;
}

/* ------------------------------------------------------------------ */
/* Dual-level error-bound controller, Algorithm 1.                     */
/*   table-wise: class from eta and two thresholds                     */
/*       eta > S_EMB_hindex -> small ; eta < L_EMB_hindex -> large ;   */
/*       otherwise medium                                              */
/*       LargeEB = GlobalEB*alpha, SmallEB = GlobalEB/beta,            */
/*       MediumEB = GlobalEB                                           */
/*   iteration-wise: multiplier m(i) over the initial phase            */
/*       stepwise (default, Section III-C): staircase from M0 to 1     */
/*       in `steps` equal drops over `decay_len` iterations            */
/*       drop (the comparison method of Section IV-B): M0 until the    */
/*       end of the phase, then 1                                      */
/* Readings: thresholds are caller-supplied; the staircase is given in */
/* closed form of the iteration (equal to Algorithm 1's compounding    */
/* update with DecayFunc(i) = m(i)/m(i-1)); RANGE_REL mode, clamp and  */
/* relative floor are extensions the synthetic workloads need.         */
/* ------------------------------------------------------------------ */
typedef struct {
    int32_t mode;       /* 0: absolute (paper); 1: global_eb is a fraction of (max-min) */
    int32_t decay_kind; /* 0 none, 1 stepwise, 2 drop */
    double global_eb, alpha, beta;
    double h_large, h_small;
    int64_t decay_start, decay_len;
    int32_t decay_steps;
    int32_t reserved;
    double decay_mult0;
    double eb_min, eb_max; /* applied when > 0 */
    double rel_floor;      /* when > 0: eb >= rel_floor*(max-min) */
} orc_controller_params;

#define ORC_CLASS_SMALL 0
#define ORC_CLASS_MEDIUM 1
#define ORC_CLASS_LARGE 2

int orc_classify(double eta, double h_large, double h_small) {
    if (eta > h_small) return ORC_CLASS_SMALL;
    if (eta < h_large) return ORC_CLASS_LARGE;
    return ORC_CLASS_MEDIUM;
}

double orc_decay_multiplier(const orc_controller_params* p, int64_t i) {
    if (p->decay_kind == 0 || p->decay_len <= 0) return 1.0;
    if (i >= p->decay_start + p->decay_len) return 1.0;
    if (p->decay_kind == 2) return p->decay_mult0;
    if (i < p->decay_start) return p->decay_mult0;
    if (p->decay_kind == 3) /* linear */
        return p->decay_mult0 - (p->decay_mult0 - 1.0) * (double)(i - p->decay_start) / (double)p->decay_len;
    if (p->decay_kind == 4) /* logarithmic: fast at first, then slow */
        return p->decay_mult0 -
               (p->decay_mult0 - 1.0) * (log(1.0 + (double)(i - p->decay_start)) / log(1.0 + (double)p->decay_len));
    int64_t Ks = p->decay_steps;
    if (Ks < 1) return 1.0;
    int64_t s = ((i - p->decay_start) * Ks) / p->decay_len;
    if (s > Ks) s = Ks;
    if (s == Ks) return 1.0;
    return p->decay_mult0 - (p->decay_mult0 - 1.0) * (double)s / (double)Ks;
}

int orc_controller(const orc_table_stats* st, int T, const orc_controller_params* p, const int32_t* class_override,
                   int64_t iteration, float* eb_out, int32_t* class_out) {
    if (!st || !p || !eb_out || T < 1) return ORC_EINVAL;
    double m = orc_decay_multiplier(p, iteration);
    for (int t = 0; t < T; ++t) {
        double eta = orc_homo_index(st[t].n_unique_raw, st[t].n_unique_quant);
        int cls = orc_classify(eta, p->h_large, p->h_small);
        if (class_override && class_override[t] >= 0) cls = class_override[t];
        double range = (double)st[t].max - (double)st[t].min;
        double e = p->global_eb;
        if (p->mode == 1) e = p->global_eb * range;
        if (cls == ORC_CLASS_LARGE) e = e * p->alpha;
        if (cls == ORC_CLASS_SMALL) e = e / p->beta;
        e = e * m;
        if (p->eb_min > 0.0 && e < p->eb_min) e = p->eb_min;
        if (p->eb_max > 0.0 && e > p->eb_max) e = p->eb_max;
        if (p->rel_floor > 0.0) {
            double f = p->rel_floor * range;
            if (e < f) e = f;
        }
        eb_out[t] = (float)e;
        if (class_out) class_out[t] = cls;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* Container (a reading throughout; Section III-E only asks for one    */
/* buffer holding all tables, chunked so that decoding is parallel,    */
/* with every write offset known before the write, and Section III-A   */
/* for size metadata).                                                 */
/*                                                                     */
/* A table's n = B*D symbols (row-major) are cut into groups of W*S    */
/* symbols.  Inside a group the W chunks take turns: chunk l gets      */
/* symbols  g*W*S + j*W*V + l*V + v  for j = 0.., v = 0..V-1, in that  */
/* order, as far as they are < n.  A chunk's codewords are packed      */
/* MSB-first into little-endian 32-bit words (stream bit k is bit      */
/* 31-(k%32) of word k/32) and zero-padded to a whole word.  A group   */
/* occupies consecutive words: its W chunks in order, then one record  */
/* of two words (index in table, raw bits) per escape of the group,    */
/* in increasing index.  Groups follow one another: table 0 group 0,   */
/* group 1, ... then table 1.  So every offset is a prefix sum over    */
/* groups.                                                             */
/*                                                                     */
/* bytes   0..127  header (u32 magic, version, dtype, T, B, D, R, S,   */
/*                 LMAX, W, V, n_groups_total; u64 n_outliers_total,   */
/*                 payload_words_total, off_group, off_chunk,          */
/*                 off_payload, off_codebook, total_bytes; 24 zero     */
/*                 bytes)                                              */
/* then T directory entries of 56 bytes (u32 eb bits, n_used, sym_lo,  */
/*                 sym_hi, n_outliers, n_groups; u64 codebook_off, 0,  */
/*                 payload_word_off, payload_words)                    */
/* off_group       u32 first word (relative to off_payload) per group  */
/* off_chunk       u8 word count per chunk, W per group                */
/* off_payload     the words (chunks and escape records)               */
/* off_codebook    per table u8 length[sym_lo..sym_hi] (0 = unused),   */
/*                 each block zero-padded to 4 bytes                   */
/* Sections start 16-byte aligned; the first three have sizes that     */
/* depend on the geometry alone.                                       */
/* ------------------------------------------------------------------ */
static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static void put32(uint8_t* p, uint32_t v) { memcpy(p, &v, 4); }
static void put64(uint8_t* p, uint64_t v) { memcpy(p, &v, 8); }
static uint32_t get32(const uint8_t* p) {
    uint32_t v;
    memcpy(&v, p, 4);
    return v;
}
static uint64_t get64(const uint8_t* p) {
    uint64_t v;
    memcpy(&v, p, 8);
    return v;
}

/* index in the table of the k-th symbol of chunk l of group g */
static size_t chunk_symbol_index(size_t g, uint32_t l, uint32_t k, uint32_t S) {
    return g * (size_t)ORC_W * S + (size_t)(k / ORC_V) * (ORC_W * ORC_V) + (size_t)l * ORC_V + (k % ORC_V);
}

static int check_geometry(int dtype, int T, int64_t B, int64_t D, int R, int S, int LMAX) {
    if (dtype != ORC_F32 && dtype != ORC_F16) return ORC_EINVAL;
    if (T < 1 || B < 1 || D < 1) return ORC_EINVAL;
    if ((uint64_t)B * (uint64_t)D > 0x7FFFFFFFull) return ORC_EINVAL;
    if (R < 2 || R > 2048 || (R & (R - 1))) return ORC_EINVAL;
    if (LMAX < 1 || LMAX > ORC_LMAX_LIMIT || (1 << LMAX) < 2 * R) return ORC_EINVAL;
    if (S < (int)ORC_V || S % (int)ORC_V) return ORC_EINVAL;
    if ((int64_t)S * LMAX > 255 * 32) return ORC_EINVAL; /* word count of a chunk is a u8 */
    return ORC_OK;
}

size_t orc_compress_bound(int dtype, int T, int64_t B, int64_t D, int R, int S, int LMAX) {
    if (check_geometry(dtype, T, B, D, R, S, LMAX) != ORC_OK) return 0;
    size_t n = (size_t)B * (size_t)D;
    size_t G = (n + (size_t)ORC_W * S - 1) / ((size_t)ORC_W * S);
    size_t NG = G * (size_t)T;
    size_t off = align_up(ORC_HEADER_BYTES + (size_t)ORC_DIR_BYTES * T, 16);
    off = align_up(off + 4 * NG, 16);
    off = align_up(off + ORC_W * NG, 16);
    size_t words_per_chunk = ((size_t)S * LMAX + 31) / 32;
    off = align_up(off + 4 * words_per_chunk * ORC_W * NG + 8 * n * T, 16); /* every chunk full, every element an escape */
    return off + (size_t)T * align_up(2 * (size_t)R, 4);
}

typedef struct {
    uint8_t len[4096];
    uint32_t code[4096];
    int n_used, sym_lo, sym_hi;
    uint32_t n_outliers;
    uint32_t* out_idx;
    uint32_t* out_raw;
    uint8_t* chunk_words; /* W per group */
    uint64_t* group_word; /* first word of each group, relative to the table */
    uint32_t* words;      /* chunks and escape records of all groups */
    uint64_t n_words;
    uint32_t* ref;        /* row matching: first row of the batch with this row's content (NULL: not used) */
} orc_table_work;

static void free_table_work(orc_table_work* w, int T) {
    if (!w) return;
    for (int t = 0; t < T; ++t) {
        free(w[t].out_idx);
        free(w[t].out_raw);
        free(w[t].chunk_words);
        free(w[t].group_word);
        free(w[t].words);
        free(w[t].ref);
    }
    free(w);
}

/*
 * carry_hist (optional, T*K counts): code table t with the Huffman codebook of carry_hist[t] -- the symbol counts of
 * an EARLIER payload -- instead of its own (the value distributions change little between training iterations,
 * Section IV-C, so the previous iteration's codebook fits the next one).  Readings, the paper being silent:
 *   - the count of symbol 0 (the escape) is raised by one before the codebook is built, so that an escape can always
 *     be coded;
 *   - a symbol the carried counts do not contain is stored as an escape (symbol 0 in the stream plus a record with
 *     the raw value), so the bound holds for any payload.
 * hist_out (optional, T*K): the symbol counts of THIS payload (before that substitution), i.e. what the next call
 * would be given as carry_hist.
 */
/* rows of one table as sequences of element identities (symbol, or raw bits for an escape), for the row matching */
static const uint64_t* g_ident;
static size_t g_ident_D;
static int ident_row_cmp(const void* a, const void* b) {
    uint32_t ia = *(const uint32_t*)a, ib = *(const uint32_t*)b;
    int c = memcmp(g_ident + (size_t)ia * g_ident_D, g_ident + (size_t)ib * g_ident_D, g_ident_D * sizeof(uint64_t));
    if (c) return c;
    return ia < ib ? -1 : (ia > ib ? 1 : 0);
}

/*
 * row_match (optional, T flags): tables flagged here are coded with the vector-based LZ step of Section III-D
 * before the entropy coder: a row (embedding vector) that equals an earlier row of the same table in the batch is
 * not coded at all; it carries a reference to that row.  Readings, the paper giving the idea but no format:
 *   - the fixed pattern is one whole row, compared after quantisation: two rows are equal when all their symbols
 *     are, and, where a symbol is the escape, the raw bits too;
 *   - the window is the whole batch and the reference is always the FIRST row of the batch with that content, so a
 *     referenced row is always a coded one (no chains) and the decoder can copy rows in parallel;
 *   - the references are stored as u32 ref[B] (ref[i] = i for a coded row) behind the code-length blocks, 16-byte
 *     aligned, the directory entry's second u64 giving the byte offset (0 for a table without row matching);
 *   - the elements of a referencing row take no part in histogram, codebook, chunk bits or escape records.
 */
static int compress_impl(const void* payload, int dtype, int T, int64_t B, int64_t D, int R, int S, int LMAX,
                         const float* eb, uint8_t* out, size_t capacity, uint64_t* out_bytes /* 1 + T */,
                         const uint64_t* carry_hist, uint64_t* hist_out, const uint8_t* row_match) {
    int rc = check_geometry(dtype, T, B, D, R, S, LMAX);
    if (rc != ORC_OK) return rc;
    if (!payload || !eb || !out || !out_bytes) return ORC_EINVAL;
    for (int t = 0; t < T; ++t)
        if (!(eb[t] > 0.0f) || isinf(eb[t])) return ORC_EINVAL;
    const int K = 2 * R;
    const size_t es = dtype == ORC_F16 ? 2 : 4;
    const size_t n = (size_t)B * (size_t)D;
    const size_t GS = (size_t)ORC_W * (size_t)S;
    const size_t G = (n + GS - 1) / GS;

    orc_table_work* work = (orc_table_work*)calloc((size_t)T, sizeof(orc_table_work));
    uint16_t* sym = (uint16_t*)malloc(sizeof(uint16_t) * n);
    uint64_t* hist = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)K);
    if (!work || !sym || !hist) {
        free(sym);
        free(hist);
        free_table_work(work, T);
        return ORC_ENOMEM;
    }

    for (int t = 0; t < T; ++t) {
        orc_table_work* w = &work[t];
        const uint8_t* tab = (const uint8_t*)payload + (size_t)t * n * es;
        /* quantise, collect escapes in index order */
        orc_quantize(tab, dtype, n, eb[t], R, sym, NULL);
        if (row_match && row_match[t]) {
            uint64_t* ident = (uint64_t*)malloc(sizeof(uint64_t) * n);
            uint32_t* order = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)B);
            w->ref = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)B);
            if (!ident || !order || !w->ref) {
                free(ident);
                free(order);
                free(sym);
                free(hist);
                free_table_work(work, T);
                return ORC_ENOMEM;
            }
            for (size_t i = 0; i < n; ++i) ident[i] = sym[i] ? (uint64_t)sym[i] : ((1ull << 32) | load_raw(tab, dtype, i));
            for (int64_t r = 0; r < B; ++r) order[r] = (uint32_t)r;
            g_ident = ident;
            g_ident_D = (size_t)D;
            qsort(order, (size_t)B, sizeof(uint32_t), ident_row_cmp);
            for (int64_t k = 0; k < B; ++k) { /* equal rows are adjacent, the smallest index first */
                if (k > 0 && memcmp(ident + (size_t)order[k] * D, ident + (size_t)order[k - 1] * D, (size_t)D * sizeof(uint64_t)) == 0)
                    w->ref[order[k]] = w->ref[order[k - 1]];
                else
                    w->ref[order[k]] = order[k];
            }
            for (int64_t r = 0; r < B; ++r)
                if (w->ref[r] != (uint32_t)r)
                    for (int64_t e = 0; e < D; ++e) sym[(size_t)r * D + e] = 0xFFFF; /* not coded */
            free(ident);
            free(order);
        }
        /* histogram and codebook (elements of referencing rows do not count) */
        memset(hist, 0, sizeof(uint64_t) * (size_t)K);
        for (size_t i = 0; i < n; ++i)
            if (sym[i] != 0xFFFF) hist[sym[i]]++;
        if (hist_out) memcpy(hist_out + (size_t)t * K, hist, sizeof(uint64_t) * (size_t)K);
        if (carry_hist) {
            memcpy(hist, carry_hist + (size_t)t * K, sizeof(uint64_t) * (size_t)K);
            hist[0] += 1;
            for (size_t i = 0; i < n; ++i)
                if (sym[i] != 0xFFFF && hist[sym[i]] == 0) sym[i] = 0; /* no code for it: an escape */
        }
        orc_codebook(hist, K, LMAX, w->len, w->code, &w->n_used, NULL);
        w->sym_lo = -1;
        for (int k = 0; k < K; ++k)
            if (hist[k]) {
                if (w->sym_lo < 0) w->sym_lo = k;
                w->sym_hi = k;
            }
        size_t n_out = 0;
        for (size_t i = 0; i < n; ++i) n_out += sym[i] == 0;
        w->n_outliers = (uint32_t)n_out;
        w->out_idx = (uint32_t*)malloc(sizeof(uint32_t) * (n_out ? n_out : 1));
        w->out_raw = (uint32_t*)malloc(sizeof(uint32_t) * (n_out ? n_out : 1));
        size_t o = 0;
        for (size_t i = 0; i < n; ++i)
            if (sym[i] == 0) {
                w->out_idx[o] = (uint32_t)i;
                w->out_raw[o] = load_raw(tab, dtype, i);
                o++;
            }
        /* chunk sizes and group offsets: a group = its chunks' words, then two words per escape */
        w->chunk_words = (uint8_t*)calloc(G * ORC_W, 1);
        w->group_word = (uint64_t*)calloc(G, sizeof(uint64_t));
        uint64_t total_words = 0;
        for (size_t g = 0; g < G; ++g) {
            w->group_word[g] = total_words;
            for (uint32_t l = 0; l < ORC_W; ++l) {
                uint64_t bits = 0;
                for (uint32_t k = 0; k < (uint32_t)S; ++k) {
                    size_t idx = chunk_symbol_index(g, l, k, (uint32_t)S);
                    if (idx < n && sym[idx] != 0xFFFF) bits += w->len[sym[idx]];
                }
                uint64_t nw = (bits + 31) / 32;
                w->chunk_words[g * ORC_W + l] = (uint8_t)nw;
                total_words += nw;
            }
            size_t lo = g * GS, hi = lo + GS < n ? lo + GS : n;
            for (size_t i = lo; i < hi; ++i) total_words += 2 * (sym[i] == 0);
        }
        w->n_words = total_words;
        w->words = (uint32_t*)calloc(total_words ? total_words : 1, sizeof(uint32_t));
        /* bit packing, then the group's escape records */
        uint64_t wpos = 0;
        size_t o2 = 0;
        for (size_t g = 0; g < G; ++g) {
            for (uint32_t l = 0; l < ORC_W; ++l) {
                uint64_t bit = 0; /* bit position inside the chunk */
                for (uint32_t k = 0; k < (uint32_t)S; ++k) {
                    size_t idx = chunk_symbol_index(g, l, k, (uint32_t)S);
                    if (idx >= n || sym[idx] == 0xFFFF) continue;
                    uint32_t L = w->len[sym[idx]];
                    uint32_t c = w->code[sym[idx]];
                    for (uint32_t b = 0; b < L; ++b) { /* MSB of the codeword first */
                        uint32_t v = (c >> (L - 1 - b)) & 1u;
                        if (v) w->words[wpos + bit / 32] |= 1u << (31 - (bit % 32));
                        bit++;
                    }
                }
                wpos += w->chunk_words[g * ORC_W + l];
            }
            size_t hi = (g + 1) * GS < n ? (g + 1) * GS : n;
            while (o2 < w->n_outliers && w->out_idx[o2] < hi) { /* out_idx is increasing */
                w->words[wpos++] = w->out_idx[o2];
                w->words[wpos++] = w->out_raw[o2];
                o2++;
            }
        }
    }
    free(sym);
    free(hist);

    /* layout */
    const size_t NG = G * (size_t)T;
    size_t off_group = align_up(ORC_HEADER_BYTES + (size_t)ORC_DIR_BYTES * T, 16);
    size_t off_chunk = align_up(off_group + 4 * NG, 16);
    size_t off_payload = align_up(off_chunk + ORC_W * NG, 16);
    uint64_t n_out_total = 0, words_total = 0;
    for (int t = 0; t < T; ++t) {
        n_out_total += work[t].n_outliers;
        words_total += work[t].n_words;
    }
    size_t off_codebook = align_up(off_payload + 4 * (size_t)words_total, 16);
    size_t cur = off_codebook;
    size_t* cb_off = (size_t*)malloc(sizeof(size_t) * (size_t)T);
    for (int t = 0; t < T; ++t) {
        cb_off[t] = cur;
        cur += align_up((size_t)(work[t].sym_hi - work[t].sym_lo + 1), 4);
    }
    /* row references of the tables that use row matching, behind the code-length blocks */
    size_t* ref_off = (size_t*)calloc((size_t)T, sizeof(size_t));
    for (int t = 0; t < T; ++t)
        if (work[t].ref) {
            cur = align_up(cur, 16);
            ref_off[t] = cur;
            cur += 4 * (size_t)B;
        }
    size_t total = cur;
    if (words_total > 0xFFFFFFFFull) {
        free(ref_off);
        free(cb_off);
        free_table_work(work, T);
        return ORC_EINVAL;
    }
    if (total > capacity) {
        free(cb_off);
        free(ref_off);
        free_table_work(work, T);
        out_bytes[0] = 0;
        return ORC_ECAPACITY;
    }
    memset(out, 0, total);
    put32(out + 0, ORC_MAGIC);
    put32(out + 4, ORC_VERSION);
    put32(out + 8, (uint32_t)dtype);
    put32(out + 12, (uint32_t)T);
    put32(out + 16, (uint32_t)B);
    put32(out + 20, (uint32_t)D);
    put32(out + 24, (uint32_t)R);
    put32(out + 28, (uint32_t)S);
    put32(out + 32, (uint32_t)LMAX);
    put32(out + 36, ORC_W);
    put32(out + 40, ORC_V);
    put32(out + 44, (uint32_t)NG);
    put64(out + 48, n_out_total);
    put64(out + 56, words_total);
    put64(out + 64, off_group);
    put64(out + 72, off_chunk);
    put64(out + 80, off_payload);
    put64(out + 88, off_codebook);
    put64(out + 96, total);
    uint64_t word_base = 0;
    for (int t = 0; t < T; ++t) {
        orc_table_work* w = &work[t];
        uint8_t* d = out + ORC_HEADER_BYTES + (size_t)ORC_DIR_BYTES * t;
        uint32_t ebbits;
        memcpy(&ebbits, &eb[t], 4);
        put32(d + 0, ebbits);
        put32(d + 4, (uint32_t)w->n_used);
        put32(d + 8, (uint32_t)w->sym_lo);
        put32(d + 12, (uint32_t)w->sym_hi);
        put32(d + 16, w->n_outliers);
        put32(d + 20, (uint32_t)G);
        put64(d + 24, cb_off[t]);
        put64(d + 32, ref_off[t]);
        put64(d + 40, word_base);
        put64(d + 48, w->n_words);
        memcpy(out + cb_off[t], w->len + w->sym_lo, (size_t)(w->sym_hi - w->sym_lo + 1));
        for (size_t g = 0; g < G; ++g)
            put32(out + off_group + 4 * ((size_t)t * G + g), (uint32_t)(word_base + w->group_word[g]));
        memcpy(out + off_chunk + ORC_W * (size_t)t * G, w->chunk_words, ORC_W * G);
        memcpy(out + off_payload + 4 * word_base, w->words, 4 * (size_t)w->n_words);
        /* bytes attributable to this table (size metadata of the pipeline's second stage) */
        out_bytes[1 + t] = 4 * w->n_words + align_up((size_t)(w->sym_hi - w->sym_lo + 1), 4) + (ORC_W + 4) * G +
                           ORC_DIR_BYTES;
        if (w->ref) {
            for (int64_t r = 0; r < B; ++r) put32(out + ref_off[t] + 4 * (size_t)r, w->ref[r]);
            out_bytes[1 + t] += 4 * (uint64_t)B;
        }
        word_base += w->n_words;
    }
    out_bytes[0] = total;
    free(cb_off);
    free(ref_off);
    free_table_work(work, T);
    return ORC_OK;
}

int orc_compress(const void* payload, int dtype, int T, int64_t B, int64_t D, int R, int S, int LMAX,
                 const float* eb, uint8_t* out, size_t capacity, uint64_t* out_bytes /* 1 + T */) {
    return compress_impl(payload, dtype, T, B, D, R, S, LMAX, eb, out, capacity, out_bytes, NULL, NULL, NULL);
}

int orc_compress_carried(const void* payload, int dtype, int T, int64_t B, int64_t D, int R, int S, int LMAX,
                         const float* eb, uint8_t* out, size_t capacity, uint64_t* out_bytes /* 1 + T */,
                         const uint64_t* carry_hist /* T*K or NULL */, uint64_t* hist_out /* T*K or NULL */) {
    return compress_impl(payload, dtype, T, B, D, R, S, LMAX, eb, out, capacity, out_bytes, carry_hist, hist_out, NULL);
}

int orc_compress_rows(const void* payload, int dtype, int T, int64_t B, int64_t D, int R, int S, int LMAX,
                      const float* eb, uint8_t* out, size_t capacity, uint64_t* out_bytes /* 1 + T */,
                      const uint8_t* row_match /* T flags */) {
    return compress_impl(payload, dtype, T, B, D, R, S, LMAX, eb, out, capacity, out_bytes, NULL, NULL, row_match);
}

/* ------------------------------------------------------------------ */
/* Compressor selection (Section III-D "Selection Between Two          */
/* Encoders", Eq. 2, Algorithm "Compressor Selection").                */
/* ------------------------------------------------------------------ */
/* Eq. 2: the speed-up of compress + send + decompress over sending raw, for compression ratio cr, network
 * bandwidth net and compression / decompression throughputs tc, td (one unit for all three).  0 when an
 * argument is not positive. */
double orc_speedup(double cr, double net, double tc, double td) {
    if (!(cr > 0.0) || !(net > 0.0) || !(tc > 0.0) || !(td > 0.0)) return 0.0;
    return 1.0 / (1.0 / cr + net * (1.0 / tc + 1.0 / td));
}

/* The algorithm's loop over tables with the speed-ups already estimated from a sample: cr is [n_comp][T]
 * (compressor-major), tc and td are [n_comp].  Per table the compressor with the largest estimate wins; between
 * equal estimates the one listed first.  choice[t] gets its index, best[t] (optional) its estimate. */
int orc_select(int T, int n_comp, const double* cr, const double* tc, const double* td, double net, int32_t* choice,
               double* best) {
    if (T < 1 || n_comp < 1 || !cr || !tc || !td || !choice) return ORC_EINVAL;
    for (int t = 0; t < T; ++t) {
        int arg = 0;
        double top = orc_speedup(cr[t], net, tc[0], td[0]);
        for (int c = 1; c < n_comp; ++c) {
            double s = orc_speedup(cr[(size_t)c * T + t], net, tc[c], td[c]);
            if (s > top) {
                top = s;
                arg = c;
            }
        }
        choice[t] = arg;
        if (best) best[t] = top;
    }
    return ORC_OK;
}

/* The whole procedure on a sampled payload with the two compressors of this path: 0 = the entropy coder alone,
 * 1 = the vector-based LZ step (row matching) in front of it.  Both compress the sample at the given bounds; a
 * table's ratio under a compressor is its uncompressed bytes over the bytes the container attributes to it. */
int orc_select_compressors(const void* payload, int dtype, int T, int64_t B, int64_t D, int R, int S, int LMAX,
                           const float* eb, double net, const double* tc /* 2 */, const double* td /* 2 */,
                           int32_t* choice /* T */, double* best /* T, optional */) {
    if (!payload || !eb || !tc || !td || !choice || T < 1) return ORC_EINVAL;
    size_t cap = orc_compress_bound(dtype, T, B, D, R, S, LMAX);
    if (cap == 0) return ORC_EINVAL;
    cap += (size_t)T * (16 + 4 * (size_t)B) + 16;
    uint8_t* out = (uint8_t*)malloc(cap);
    uint64_t* sizes = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(1 + T));
    uint8_t* flags = (uint8_t*)malloc((size_t)T);
    double* cr = (double*)malloc(sizeof(double) * 2 * (size_t)T);
    int rc = (out && sizes && flags && cr) ? ORC_OK : ORC_ENOMEM;
    const double raw = (double)B * (double)D * (dtype == ORC_F16 ? 2.0 : 4.0);
    for (int c = 0; c < 2 && rc == ORC_OK; ++c) {
        memset(flags, c, (size_t)T);
        rc = orc_compress_rows(payload, dtype, T, B, D, R, S, LMAX, eb, out, cap, sizes, flags);
        for (int t = 0; t < T && rc == ORC_OK; ++t) cr[(size_t)c * T + t] = raw / (double)sizes[1 + t];
    }
    if (rc == ORC_OK) rc = orc_select(T, 2, cr, tc, td, net, choice, best);
    free(out);
    free(sizes);
    free(flags);
    free(cr);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Decoder: mirrors the container; bit-by-bit canonical decoding with  */
/* the first code of each length (no lookup table).                    */
/* ------------------------------------------------------------------ */
int orc_container_info(const uint8_t* comp, size_t bytes, uint32_t* fields12, uint64_t* fields8) {
    if (!comp || bytes < ORC_HEADER_BYTES) return ORC_ECORRUPT;
    if (get32(comp) != ORC_MAGIC || get32(comp + 4) != ORC_VERSION) return ORC_ECORRUPT;
    for (int i = 0; i < 12; ++i) fields12[i] = get32(comp + 4 * i);
    for (int i = 0; i < 8; ++i) fields8[i] = get64(comp + 48 + 8 * i);
    return ORC_OK;
}

int orc_decompress(const uint8_t* comp, size_t bytes, void* out, size_t out_capacity_bytes,
                   uint16_t* sym_out /* optional, T*B*D */) {
    uint32_t f[12];
    uint64_t q[8];
    int rc = orc_container_info(comp, bytes, f, q);
    if (rc != ORC_OK) return rc;
    int dtype = (int)f[2], T = (int)f[3];
    int64_t B = f[4], D = f[5];
    int R = (int)f[6], S = (int)f[7], LMAX = (int)f[8];
    if (f[9] != ORC_W || f[10] != ORC_V) return ORC_ECORRUPT;
    if (check_geometry(dtype, T, B, D, R, S, LMAX) != ORC_OK) return ORC_ECORRUPT;
    const int K = 2 * R;
    const size_t es = dtype == ORC_F16 ? 2 : 4;
    const size_t n = (size_t)B * (size_t)D;
    const size_t GS = (size_t)ORC_W * (size_t)S;
    const size_t G = (n + GS - 1) / GS;
    const size_t NG = G * (size_t)T;
    uint64_t n_out_total = q[0], words_total = q[1];
    uint64_t off_group = q[2], off_chunk = q[3], off_payload = q[4], off_codebook = q[5], total = q[6];
    if (f[11] != NG) return ORC_ECORRUPT;
    if (total > bytes) return ORC_ECORRUPT;
    if (off_group != align_up(ORC_HEADER_BYTES + (size_t)ORC_DIR_BYTES * T, 16)) return ORC_ECORRUPT;
    if (off_chunk != align_up(off_group + 4 * NG, 16)) return ORC_ECORRUPT;
    if (off_payload != align_up(off_chunk + ORC_W * NG, 16)) return ORC_ECORRUPT;
    if (words_total > 0xFFFFFFFFull || n_out_total > (uint64_t)n * T) return ORC_ECORRUPT;
    if (off_codebook != align_up(off_payload + 4 * words_total, 16)) return ORC_ECORRUPT;
    /* (every table has a code-length block, padded to four bytes) */
    if (total < off_codebook || total - off_codebook < 4) return ORC_ECORRUPT;
    if (!out || out_capacity_bytes < n * T * es) return ORC_ECAPACITY;

    uint64_t n_out_tables = 0; /* the header's escape count is the sum of the tables' */
    for (int t = 0; t < T; ++t) n_out_tables += get32(comp + ORC_HEADER_BYTES + (size_t)ORC_DIR_BYTES * t + 16);
    if (n_out_tables != n_out_total) return ORC_ECORRUPT;
    for (int t = 0; t < T; ++t) {
        const uint8_t* d = comp + ORC_HEADER_BYTES + (size_t)ORC_DIR_BYTES * t;
        float eb;
        uint32_t ebbits = get32(d);
        memcpy(&eb, &ebbits, 4);
        uint32_t n_used = get32(d + 4), sym_lo = get32(d + 8), sym_hi = get32(d + 12);
        uint32_t n_outl = get32(d + 16);
        uint64_t cb_off = get64(d + 24);
        uint64_t ref_off = get64(d + 32); /* row matching: u32 ref[B], 0 = none */
        if (ref_off) {
            /* (written without additions: an offset near 2^64 must not wrap past the test) */
            if (ref_off % 4 || ref_off < off_codebook || ref_off > total || 4 * (uint64_t)B > total - ref_off) return ORC_ECORRUPT;
            for (int64_t r = 0; r < B; ++r) { /* a reference points back to a coded row */
                uint32_t o = get32(comp + ref_off + 4 * (size_t)r);
                if (o > (uint32_t)r || get32(comp + ref_off + 4 * (size_t)o) != o) return ORC_ECORRUPT;
            }
        }
        if (!(eb > 0.0f) || isinf(eb)) return ORC_ECORRUPT;
        if (get32(d + 20) != G) return ORC_ECORRUPT;
        if (sym_lo > sym_hi || sym_hi >= (uint32_t)K || n_used < 1 || n_used > sym_hi - sym_lo + 1) return ORC_ECORRUPT;
        if (cb_off < off_codebook || cb_off > total || (uint64_t)(sym_hi - sym_lo + 1) > total - cb_off) return ORC_ECORRUPT;
        uint64_t seen_outl = 0;
        orc_qparam qp = make_qparam(eb);

        /* rebuild canonical code from lengths */
        uint8_t len[4096];
        memset(len, 0, sizeof len);
        uint32_t count_len[ORC_LMAX_LIMIT + 2];
        memset(count_len, 0, sizeof count_len);
        uint32_t used = 0;
        for (uint32_t k = sym_lo; k <= sym_hi; ++k) {
            len[k] = comp[cb_off + (k - sym_lo)];
            if (len[k] > LMAX) return ORC_ECORRUPT;
            if (len[k]) {
                count_len[len[k]]++;
                used++;
            }
        }
        /* symbols of each length in increasing order; first code per length */
        uint32_t first_code[ORC_LMAX_LIMIT + 2], first_index[ORC_LMAX_LIMIT + 2];
        uint16_t sorted[4096];
        if (n_used == 1) {
            if (used != 0 || sym_lo != sym_hi) return ORC_ECORRUPT;
        } else {
            if (used != n_used) return ORC_ECORRUPT;
            uint64_t kraft = 0;
            for (int L = 1; L <= LMAX; ++L) kraft += (uint64_t)count_len[L] << (LMAX - L);
            if (kraft != (1ull << LMAX)) return ORC_ECORRUPT;
            uint32_t codev = 0, idx = 0;
            for (int L = 1; L <= LMAX; ++L) {
                codev <<= 1;
                first_code[L] = codev;
                first_index[L] = idx;
                for (uint32_t k = sym_lo; k <= sym_hi; ++k)
                    if (len[k] == L) sorted[idx++] = (uint16_t)k;
                codev += count_len[L];
            }
        }
        uint8_t* tab_out = (uint8_t*)out + (size_t)t * n * es;
        for (size_t g = 0; g < G; ++g) {
            size_t gi = (size_t)t * G + g;
            uint64_t w0 = get32(comp + off_group + 4 * gi);
            uint64_t w_end = gi + 1 < NG ? get32(comp + off_group + 4 * (gi + 1)) : words_total;
            if (w_end < w0 || w_end > words_total) return ORC_ECORRUPT;
            for (uint32_t l = 0; l < ORC_W; ++l) {
                uint32_t nw = comp[off_chunk + ORC_W * gi + l];
                if (w0 + nw > w_end) return ORC_ECORRUPT;
                const uint8_t* base = comp + off_payload + 4 * w0;
                uint64_t bit = 0;
                for (uint32_t k = 0; k < (uint32_t)S; ++k) {
                    size_t idx = chunk_symbol_index(g, l, k, (uint32_t)S);
                    if (idx >= n) continue;
                    if (ref_off) { /* a referencing row has no bits in the stream */
                        size_t row = idx / (size_t)D;
                        if (get32(comp + ref_off + 4 * row) != (uint32_t)row) {
                            if (sym_out) sym_out[(size_t)t * n + idx] = 0xFFFF;
                            continue;
                        }
                    }
                    uint32_t c;
                    if (n_used == 1) {
                        c = sym_lo;
                    } else {
                        uint32_t acc = 0;
                        int L = 0;
                        for (;;) {
                            if (bit >= 32ull * nw) return ORC_ECORRUPT;
                            uint32_t word = get32(base + 4 * (bit / 32));
                            acc = (acc << 1) | ((word >> (31 - (bit % 32))) & 1u);
                            bit++;
                            L++;
                            if (L > LMAX) return ORC_ECORRUPT;
                            if (count_len[L] && acc >= first_code[L] && acc - first_code[L] < count_len[L]) {
                                c = sorted[first_index[L] + (acc - first_code[L])];
                                break;
                            }
                        }
                    }
                    if (sym_out) sym_out[(size_t)t * n + idx] = (uint16_t)c;
                    float v = c ? dequantize_one(c, &qp, R) : 0.0f;
                    if (dtype == ORC_F16) ((uint16_t*)tab_out)[idx] = orc_float_to_half(v);
                    else ((float*)tab_out)[idx] = v;
                }
                w0 += nw;
            }
            /* the rest of the group's words are its escape records */
            if ((w_end - w0) % 2) return ORC_ECORRUPT;
            size_t lo = g * GS, hi = lo + GS < n ? lo + GS : n;
            for (; w0 < w_end; w0 += 2) {
                uint32_t idx = get32(comp + off_payload + 4 * w0);
                uint32_t raw = get32(comp + off_payload + 4 * w0 + 4);
                if (idx < lo || idx >= hi) return ORC_ECORRUPT;
                if (dtype == ORC_F16) ((uint16_t*)tab_out)[idx] = (uint16_t)raw;
                else ((uint32_t*)tab_out)[idx] = raw;
                seen_outl++;
            }
        }
        if (seen_outl != n_outl) return ORC_ECORRUPT;
        if (ref_off) /* referencing rows: copies of the rows they point to */
            for (int64_t r = 0; r < B; ++r) {
                uint32_t o = get32(comp + ref_off + 4 * (size_t)r);
                if (o != (uint32_t)r) {
                    memcpy(tab_out + (size_t)r * D * es, tab_out + (size_t)o * D * es, (size_t)D * es);
                    if (sym_out)
                        memcpy(sym_out + (size_t)t * n + (size_t)r * D, sym_out + (size_t)t * n + (size_t)o * D,
                               (size_t)D * sizeof(uint16_t));
                }
            }
    }
    return ORC_OK;
}
