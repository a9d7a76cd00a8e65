/*
 * dlc.h -- C ABI of the MI355X (gfx950) error-bounded compressor for DLRM
 * embedding-lookup payloads (arXiv 2407.04272).
 *
 * One GPU's share of the all-to-all payload -- T embedding-lookup tensors of
 * B rows x D elements, row-major, fp32 or fp16, resident in device memory --
 * is compressed into ONE device buffer plus size metadata (pipeline stages 1
 * and 2 of Section III-A; "multiple tensors into a single compressed tensor",
 * Section I), and decompressed on the receiving side (stage 4).  Per-table
 * error bounds come from sampled statistics (Eq. 1, Algorithm 1
 * OfflineAnalysis) and are tightened per iteration (Algorithm 1 OnlineDecay).
 *
 * Conventions
 *  - plain pointers and sizes only; every pointer is marked HOST or DEVICE.
 *  - device buffers are caller-owned; the library never frees or reallocates
 *    them.  A context owns its own workspace, allocated in dlc_create on the
 *    device that is current at that time.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Unless stated otherwise a call only enqueues work on that stream.
 *  - return value: DLC_OK or a negative dlc_status.  Errors that only the GPU
 *    can see (output capacity exceeded, corrupt container) are recorded in a
 *    device status word and returned by dlc_sync_status.
 *  - a context is not thread-safe; calls that share a context must be issued
 *    on one stream (or be ordered by the caller).
 */
/*
 * The container (little-endian; what dlc_compress writes and dlc_decompress reads)
 *
 *   header, 128 bytes   u32 magic "DLC2", version 2, dtype, T, B, D, R, S, LMAX, 64 (chunks per group), 4 (symbols a
 *                       chunk takes per turn), NG (groups in all);  then from byte 48, u64: escapes in all, payload words
 *                       in all, byte offsets of the group table, the chunk table, the payload, the code-length blocks, and
 *                       the total size;  24 zero bytes
 *   directory           T entries of 56 bytes: u32 bound (fp32 bits), used symbols, lowest and highest used symbol, escapes,
 *                       groups;  u64 byte offset of the table's code lengths, 0, first payload word, payload words
 *   group table         u32 first payload word of every group               (each section starts on a 16-byte boundary)
 *   chunk table         u8 words of every chunk, 64 per group
 *   payload             group after group: its 64 chunks (codewords most significant bit first in 32-bit words, each chunk
 *                       padded to a word), then its escape records (u32 element index in the table, u32 raw bits), by index
 *   code lengths        per table u8 length of every symbol from the lowest to the highest used one, padded to 4 bytes;
 *                       codewords are canonical: ordered by (length, symbol)
 *
 * A table's B*D elements are cut into groups of 64*S; chunk l of group g holds the elements
 * g*64*S + j*256 + l*4 + v  (j < S/4, v < 4) in that order.  Symbol 0 is the escape, symbol c > 0 stands for the value
 * (c - R) * 2 * bound.
 */
#ifndef DLC_H
#define DLC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dlc_ctx dlc_ctx;

enum { DLC_F32 = 0, DLC_F16 = 1 };

typedef enum {
    DLC_OK = 0,
    DLC_EINVAL = -1,    /* bad argument (null/misaligned pointer, geometry out of range, eb <= 0 or not finite) */
    DLC_ENOMEM = -2,    /* workspace allocation failed */
    DLC_ECAPACITY = -3, /* output buffer too small; nothing was written past its capacity */
    DLC_ECORRUPT = -4,  /* container fails validation */
    DLC_EHIP = -5,      /* a HIP runtime call failed */
    DLC_ESTATE = -6,    /* call order (bounds not set), or an internal invariant failed */
    DLC_ELIMIT = -7     /* a size beyond the fixed maximum of an entry point that allocates nothing */
} dlc_status;

/* Geometry and format parameters of one payload (Section III-D leaves them open). */
typedef struct {
    int32_t dtype;         /* DLC_F32 or DLC_F16 */
    int32_t num_tables;    /* T >= 1; a container's worst case (every element an escape: two words each on top of the
                              codewords) must stay below 2^32 words, which allows about 1.6e9 elements per container */
    int64_t batch;         /* B >= 1 rows per table */
    int64_t dim;           /* D >= 1 elements per row; B*D < 2^31 */
    int32_t radius;        /* R: power of two in [8, 2048]; alphabet 2R, symbol 0 = verbatim escape */
    int32_t chunk_symbols; /* S: symbols per chunk, one of 64, 128, 256 */
    int32_t max_code_len;  /* LMAX <= 12, 2^LMAX >= 2R */
    int32_t flags;         /* 0, or DLC_FLAG_* */
    int32_t num_dest;      /* destinations the payload is split over, 1..4096 (0 counts as 1); see below */
} dlc_config;

/* Per-destination buffers (Section III-E: the payload a GPU sends is cut along the batch axis, one piece per
 * receiving GPU, and the compressor writes every piece's compressed form straight into the send buffer in one
 * launch sequence).  With num_dest = n > 1:
 *   - `batch` is the number of rows of ONE destination's piece; the payload is [n][num_tables][batch][dim], i.e. the
 *     destination-major layout of an all-to-all send buffer;
 *   - dlc_compress writes n complete containers, each exactly what a context with num_dest = 1 and the same other
 *     fields would write for that piece (own code histograms and codebooks per piece, the per-table bounds shared);
 *     container d starts at byte d * stride of d_out, stride = (out_capacity / n) rounded down to a multiple of 256,
 *     and must fit into its stride.  The pieces are therefore at fixed displacements, as a variable-size all-to-all
 *     takes them; their sizes come back in d_out_bytes (see dlc_compress);
 *   - a destination that does not fit gets size 0 and DLC_ECAPACITY is recorded; the others are still valid;
 *   - dlc_set_error_bounds still takes num_tables bounds; dlc_stats wants num_dest = 1 (a table's statistics are
 *     over its whole batch);
 *   - dlc_decompress decodes n containers in one launch sequence (the receiving side of the exchange: one container
 *     from every sender): container d is expected at byte d * stride of d_comp, stride = (comp_bytes / n) rounded
 *     down to a multiple of 256 -- the layout dlc_compress writes for out_capacity = comp_bytes -- and the output
 *     is [n][num_tables][batch][dim].  Every container says in its header how long it is; one that fails
 *     validation is reported (DLC_ECORRUPT) and left undecoded, the others are decoded. */

/* dlc_config.flags (bit 0 is not used).  DLC_FLAG_STATS_WORKSPACE: dlc_create also allocates the buffers of
 * dlc_stats (about 24 bytes per row and table), so that statistics taken again in the middle of a run (periodic
 * re-classification of the tables) allocate nothing; without it the first dlc_stats call allocates them.  Goes
 * with every other flag. */
enum { DLC_FLAG_CARRY_CODEBOOK = 2, DLC_FLAG_ROW_MATCH = 4, DLC_FLAG_STATS_WORKSPACE = 8, DLC_FLAG_SAMPLE_CODEBOOK = 16 };

/* DLC_FLAG_CARRY_CODEBOOK: dlc_compress codes each table with the Huffman codebook built from the payload of the
 * PREVIOUS dlc_compress call on this context instead of from its own payload (Section IV-C: the value distributions
 * of the lookups change little from iteration to iteration).  The payload is then read once instead of twice.
 *   - The first call on a context, and the first call after dlc_set_error_bounds changed a bound, build their
 *     codebook from their own payload as without the flag (same bytes as without the flag).
 *   - A carried codebook is the Huffman codebook of the previous call's symbol counts with the count of symbol 0
 *     (the escape) raised by one, so that an escape can always be coded.
 *   - A symbol the carried codebook has no code for is stored as an escape (raw value), so the error bound holds
 *     for any payload; a payload unlike the previous one costs compression ratio, never correctness.
 *   - The container format is unchanged; dlc_decompress needs no flag.
 *   - The workspace of such a context also holds every group's words before they are put in place, with room for
 *     every group's worst case: about 2.6 times an fp32 payload in all (dlc_workspace_bytes says how much). */

/* DLC_FLAG_SAMPLE_CODEBOOK: the payload is read once as with DLC_FLAG_CARRY_CODEBOOK, but no call depends on the one
 * before it: the Huffman codebook of a table (Section III-D) is built from the symbol counts of a SAMPLE of the same
 * payload, a few whole groups of the table (a group = 64 * chunk_symbols consecutive elements):
 *   - ns groups: as many as hold 65536 elements, ceil(65536 / (64 * chunk_symbols)), but no more than a quarter of
 *     the table's groups (rounded up); they are groups 0, stride, 2 * stride, ... with stride = floor(groups / ns);
 *     a table of one group is counted whole;
 *   - the count of symbol 0 (the escape) is raised by one and a symbol the sample has not seen is stored as an escape,
 *     exactly as with a carried codebook, so the error bound holds whatever the sample missed.
 * Costs: a fraction of a percent of compression ratio where a table's symbols take bits at all; a table that is one
 * symbol throughout takes one bit per element instead of none.  Same container format, same workspace as with
 * DLC_FLAG_CARRY_CODEBOOK less the symbol plane; not together with DLC_FLAG_CARRY_CODEBOOK or DLC_FLAG_ROW_MATCH. */

/* DLC_FLAG_ROW_MATCH: the vector-based LZ step of Section III-D in front of the entropy coder.  The pattern is one
 * whole row (embedding vector): a row that equals an earlier row of its table in the batch after quantisation -- all
 * symbols and, where a symbol is the escape, the raw bits -- is not coded; the container stores a reference to the
 * FIRST such row (u32 ref[batch] per table behind the code-length blocks; the directory entry's second u64 is its
 * byte offset, 0 for a table without).  A referenced row is therefore always a coded one and the decoder copies rows
 * in parallel.  Per table: dlc_set_row_match switches it on and off (all on after dlc_create), which is what the
 * compressor selection of Section III-D (Eq. 2, dlc_speedup_estimate) decides offline.  Needs dim % 4 == 0; not
 * together with DLC_FLAG_CARRY_CODEBOOK or DLC_FLAG_SAMPLE_CODEBOOK; num_dest * num_tables <= 65535.  With num_dest > 1 rows are matched inside a
 * destination's piece (a container never refers to another).  The search hashes rows and compares every candidate
 * element by element; rows whose hashes meet are sorted out the long way, so the references are always those of the
 * definition. */

/* Per-table statistics of a sampled batch: what Eq. 1 needs, plus the value range. */
typedef struct {
    float min, max;          /* over finite elements (+inf / -inf if there are none) */
    uint64_t count;          /* B*D */
    uint32_t n_rows;         /* B */
    uint32_t n_unique_raw;   /* N_original: distinct rows, raw bit patterns */
    uint32_t n_unique_quant; /* N_compressed: distinct rows after quantisation at probe_eb */
    float probe_eb;
} dlc_table_stats;

enum { DLC_CLASS_SMALL = 0, DLC_CLASS_MEDIUM = 1, DLC_CLASS_LARGE = 2 };
/* Iteration-wise schedules (Section III-C names logarithmic and stepwise decay functions and gives only their end
 * points: mult0 x base at the start of the initial phase, base after it).  With u = (i - decay_start) / decay_len:
 *   STEPWISE  mult0 - (mult0 - 1) * floor(u * steps) / steps       (the paper's default)
 *   DROP      mult0 during the phase, 1 after it                    ("Drop_kx")
 *   LINEAR    mult0 - (mult0 - 1) * u
 *   LOG       mult0 - (mult0 - 1) * log(1 + (i - decay_start)) / log(1 + decay_len)   (fast at first, then slow)
 * All are mult0 before the phase and 1 from its end on; computed in double. */
enum { DLC_DECAY_NONE = 0, DLC_DECAY_STEPWISE = 1, DLC_DECAY_DROP = 2, DLC_DECAY_LINEAR = 3, DLC_DECAY_LOG = 4 };

/* Hyper-parameters of Algorithm 1. */
typedef struct {
    int32_t mode;        /* 0: global_eb is an absolute bound (the paper's mode); 1: a fraction of (max-min) */
    int32_t decay_kind;  /* DLC_DECAY_* ; stepwise is the paper's default (Section III-C) */
    double global_eb;    /* GlobalEB = MediumEB */
    double alpha, beta;  /* LargeEB = GlobalEB*alpha, SmallEB = GlobalEB/beta */
    double h_large;      /* L_EMB_hindex: eta < h_large -> large */
    double h_small;      /* S_EMB_hindex: eta > h_small -> small; otherwise medium */
    int64_t decay_start; /* first iteration of the initial phase */
    int64_t decay_len;   /* its length in iterations */
    int32_t decay_steps; /* number of equal drops of the staircase */
    int32_t reserved;    /* 0 */
    double decay_mult0;  /* multiplier at the start of the phase (2 = "Decay_2x"); 1 after the phase */
    double eb_min, eb_max; /* clamp, each applied when > 0 */
    double rel_floor;    /* when > 0: eb >= rel_floor*(max-min) */
} dlc_controller_params;

/* Creates a context for one geometry and allocates its device workspace (HOST call, allocates). */
int dlc_create(dlc_ctx** ctx_out /*HOST*/, const dlc_config* cfg /*HOST*/);
void dlc_destroy(dlc_ctx* ctx);

/* Worst-case container size in bytes for this geometry (every element an escape); 0 if cfg is invalid. */
size_t dlc_compress_bound(const dlc_config* cfg /*HOST*/);
/* Device workspace a context of this geometry holds (the statistics buffers excluded, also with DLC_FLAG_STATS_WORKSPACE). */
size_t dlc_workspace_bytes(const dlc_config* cfg /*HOST*/);

/*
 * Statistics reduction (Eq. 1; Algorithm 1, OfflineAnalysis: sampleData + homoIndexCal inputs).
 *   d_payload  DEVICE  [T][B][D] row-major, dtype of the context, 16-byte aligned
 *   h_probe_eb HOST    T bounds at which rows are quantised for N_compressed
 *   h_stats    HOST    T entries, caller-owned, filled on return
 * Distinct-row counts are exact (hashing, then every hash match is verified element by element).
 * Synchronises `stream` before returning.  Allocates its own workspace on first use (unless the context was created
 * with DLC_FLAG_STATS_WORKSPACE).  DLC_ESTATE on a context with
 * num_dest > 1 (a table's statistics are over its whole batch), DLC_EINVAL with more than 65535 tables.
 */
int dlc_stats(dlc_ctx* ctx, const void* d_payload, const float* h_probe_eb, dlc_table_stats* h_stats, void* stream);

/*
 * Dual-level error-bound controller (Algorithm 1: EMBClassification, LargeEB/MediumEB/SmallEB, OnlineDecay).
 *   h_stats == NULL : h_eb_inout holds T explicit bounds, taken as they are.
 *   h_stats != NULL : bounds are derived: class from eta = (N_original - N_compressed)/N_original and the two
 *                     thresholds (or from h_class_override[t] when that is >= 0), class bound from params,
 *                     times the iteration multiplier, clamp, floor; rounded once to fp32 and written to
 *                     h_eb_inout (T, HOST) and, if given, the classes to h_class_out (T, HOST).
 * The bounds are then copied to the context's device memory on `stream` (ordered before later compress calls
 * on that stream); a set of bounds equal to the one last copied on the same stream is not copied again.
 * Every bound must be finite and > 0.
 */
int dlc_set_error_bounds(dlc_ctx* ctx, const dlc_table_stats* h_stats, const dlc_controller_params* params,
                         const int32_t* h_class_override, int64_t iteration, float* h_eb_inout,
                         int32_t* h_class_out, void* stream);

/*
 * Compress (Section III-D quantisation encoder without predictor + Huffman entropy encoder; Section III-E
 * single launch sequence writing all tables into one buffer at scanned offsets).
 *   d_payload    DEVICE  [T][B][D], 16-byte aligned
 *   d_out        DEVICE  container, 16-byte aligned, `out_capacity` bytes; never written past capacity
 *   d_out_bytes  DEVICE  uint64[1+T]: [0] container bytes (0 on failure), [1+t] bytes attributable to table t.
 *                        With num_dest = n > 1: uint64[1 + n*T + n]: [0] sum of the n containers' sizes (0 if any failed),
 *                        [1 + d*T + t] table t of destination d, [1 + n*T + d] size of destination d's container
 * Asynchronous on `stream`.  DLC_ESTATE if bounds were never set.  Capacity overflow is detected on the GPU
 * before the overflowing write: d_out_bytes[0] = 0 and dlc_sync_status returns DLC_ECAPACITY.
 * Not for HIP graph capture: every call advances state kept on the host (the call counter that tags the look-back
 * records, the two codebook buffers a carrying context alternates between), which a replayed graph would not see.
 */
int dlc_compress(dlc_ctx* ctx, const void* d_payload, void* d_out, size_t out_capacity, uint64_t* d_out_bytes,
                 void* stream);

/*
 * Decompress (chunk-parallel decoding, Section III-E) a container produced for this context's geometry.
 *   d_comp        DEVICE  container, 16-byte aligned, comp_bytes long
 *   d_payload_out DEVICE  [T][B][D] in the context's dtype, 16-byte aligned, out_capacity >= T*B*D*sizeof(dtype)
 * Asynchronous on `stream`.  The container is self-describing (geometry, per-table bounds, code lengths); it is
 * validated on the GPU and a mismatch or inconsistency is reported by dlc_sync_status as DLC_ECORRUPT, in
 * which case the output holds unspecified values but no access left the two buffers.  The call keeps no state on
 * the host and enqueues kernels only, so it may be recorded into a HIP graph (with profiling off).
 */
int dlc_decompress(dlc_ctx* ctx, const void* d_comp, size_t comp_bytes, void* d_payload_out, size_t out_capacity,
                   void* stream);

/*
 * dlc_decompress for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It takes no context: the geometry comes from `cfg` (the one the container was
 * made with), and the decode kernels' workspace (status word, per-table counters, the row references' table) is a
 * fixed array inside the library, DLC_STATIC_MAX_TABLES tables' worth (about 160 KiB, held on every GPU the library
 * is loaded on until the process ends).  The call makes no hipMalloc, hipFree or other allocating call.
 *   cfg            HOST    as for dlc_create; num_tables * max(num_dest, 1) <= DLC_STATIC_MAX_TABLES, else DLC_ELIMIT
 *   d_comp, comp_bytes, d_payload_out, out_capacity   as for dlc_decompress
 *   d_status       DEVICE  int32[1], written on `stream` after the kernels: DLC_OK, or what dlc_sync_status would
 *                          have returned for this call (DLC_ECORRUPT for a container that fails validation)
 * Asynchronous on `stream`; output and status are the same as dlc_decompress's on the same container.  All calls on
 * one GPU share the one array: calls that overlap on a GPU (two streams, two threads) race and must be serialised
 * by the caller.  The first call on a device looks up the array's address there (no allocation either).
 */
#define DLC_STATIC_MAX_TABLES 4096
int dlc_decompress_static(const dlc_config* cfg, const void* d_comp, size_t comp_bytes, void* d_payload_out,
                          size_t out_capacity, int32_t* d_status, void* stream);

/* Row matching per table (contexts with DLC_FLAG_ROW_MATCH): h_flags HOST uint8[num_tables] (the same for every
 * destination), non-zero = store the table's repeated rows as references; NULL = all tables.  Synchronises `stream`. */
int dlc_set_row_match(dlc_ctx* ctx, const uint8_t* h_flags, void* stream);

/* Eq. 2: the speed-up of a transfer that compresses, sends and decompresses over sending raw, for compression ratio
 * cr, network bandwidth net_gbps and compression / decompression throughputs tc_gbps, td_gbps (same unit):
 * 1 / (1/cr + net * (1/tc + 1/td)).  0 if an argument is not positive. */
double dlc_speedup_estimate(double cr, double net_gbps, double tc_gbps, double td_gbps);

/*
 * Compressor selection (Section III-D "Selection Between Two Encoders", algorithm "Compressor Selection": offline, on
 * sampled data, per table the compressor with the largest Eq. 2 estimate).  The two compressors are 0 = the entropy
 * coder alone and 1 = the vector-based LZ step (row matching) in front of it; the context must have been created with
 * DLC_FLAG_ROW_MATCH and num_dest <= 1 (DLC_ESTATE otherwise) and its bounds must be set.
 *   d_sample     DEVICE  a sampled payload of the context's geometry, [T][B][D], 16-byte aligned
 *   d_out, out_capacity, d_out_bytes   DEVICE  as for dlc_compress (scratch for the two trial compressions; on return
 *                they hold the container of compressor 1 on every table)
 *   d_rec, rec_capacity  DEVICE  room for the decompressed sample, only used (and required) when the rates are measured
 *   net_gbps     network bandwidth B of Eq. 2
 *   h_tc_gbps, h_td_gbps  HOST  double[2]: compression and decompression throughput of compressor 0 and 1, in the unit
 *                of net_gbps; both NULL: the call measures them on the sample (three calls each way between events)
 *   h_choice_out HOST    uint8[T]: the compressor chosen for every table; ties go to compressor 0
 *   h_speedup_out HOST   double[T] or NULL: the chosen compressor's estimate
 * A table's compression ratio under a compressor is its uncompressed bytes over the bytes dlc_compress attributes to it
 * (d_out_bytes[1 + t]).  The choice is installed as by dlc_set_row_match.  Synchronises `stream`.
 */
int dlc_select_compressors(dlc_ctx* ctx, const void* d_sample, void* d_out, size_t out_capacity, uint64_t* d_out_bytes,
                           void* d_rec, size_t rec_capacity, double net_gbps, const double* h_tc_gbps, const double* h_td_gbps,
                           uint8_t* h_choice_out, double* h_speedup_out, void* stream);

/* Waits for `stream`, returns the first device-side error since the previous call (DLC_OK if none), clears it. */
int dlc_sync_status(dlc_ctx* ctx, void* stream);

/*
 * Inspection for tests (each synchronises `stream`):
 *   dlc_quantize       symbols (uint16, DEVICE, T*B*D) of d_payload at the current bounds -- the quantiser alone
 *   dlc_read_histogram the code histogram (uint32[T][2R], HOST) left by the last dlc_compress
 *   dlc_read_codebook  code lengths (uint8[T][2R]) and codewords (uint16[T][2R]) left by the last dlc_compress
 *   dlc_read_row_refs  row references (uint32[num_dest * T][B], HOST) left by the last dlc_compress
 *                      (DLC_FLAG_ROW_MATCH only)
 *   dlc_set_row_hash_multipliers  replaces the multipliers of the row hash that the row search uses (uint32[dim / 4][8],
 *                      HOST; DLC_FLAG_ROW_MATCH only).  The references do not depend on them; with all of them zero
 *                      every row has the same hash, which is how the tests reach the handling of equal hashes
 * With DLC_FLAG_CARRY_CODEBOOK the histogram is still that of the last call's payload, and the codebook is the one
 * built from it for the NEXT call (escape count raised by one), not the one the last call's container was coded with.
 * With DLC_FLAG_SAMPLE_CODEBOOK the histogram holds the counts of the last call's sampled groups only, and the codebook
 * is the one built from them (escape count raised by one), which the last call's container was coded with.
 */
int dlc_quantize(dlc_ctx* ctx, const void* d_payload, uint16_t* d_symbols, void* stream);
int dlc_read_histogram(dlc_ctx* ctx, uint32_t* h_hist, void* stream);
int dlc_read_codebook(dlc_ctx* ctx, uint8_t* h_len, uint16_t* h_code, void* stream);
int dlc_read_row_refs(dlc_ctx* ctx, uint32_t* h_ref, void* stream);
int dlc_set_row_hash_multipliers(dlc_ctx* ctx, const uint32_t* h_mult, void* stream);

/*
 * Kernel timing with HIP events on the caller's stream.
 *   dlc_profile_enable  level 0 off; 1 = the dominant kernel of each direction (encode, decode); 2 = every
 *                       kernel.  Each timed kernel costs two event records per call (a few microseconds).
 *   dlc_profile_read    synchronises, returns the number of kernel slots; for slot i < max_slots:
 *                       names[i] (static string), total_ms[i], launches[i]; then resets the counters
 */
int dlc_profile_enable(dlc_ctx* ctx, int level);
int dlc_profile_read(dlc_ctx* ctx, int max_slots, const char** names, float* total_ms, int32_t* launches);

const char* dlc_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* DLC_H */
