// Internal declarations shared by the HIP sources of libdlc (gfx950 only).
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dlc.h"

namespace dlc {

// ---- container constants (byte layout of the compressed buffer) -----------------------------
constexpr uint32_t kW = 64;  // chunks per group = lanes of one wavefront
constexpr uint32_t kV = 4;   // consecutive symbols a chunk takes per turn = one 16-byte fp32 load per lane
constexpr uint32_t kMagic = 0x32434C44u;  // "DLC2"
constexpr uint32_t kVersion = 2u;
constexpr uint32_t kHeaderBytes = 128;
constexpr uint32_t kDirBytes = 56;
constexpr int kLmaxLimit = 12;

// header word / qword positions
enum { H_MAGIC = 0, H_VERSION, H_DTYPE, H_T, H_B, H_D, H_R, H_S, H_LMAX, H_W, H_V, H_NG };  // u32 index
enum { HQ_NOUT = 6, HQ_WORDS, HQ_OFF_GROUP, HQ_OFF_CHUNK, HQ_OFF_PAYLOAD, HQ_OFF_CB, HQ_TOTAL };  // u64 index

struct QParam {
    float eb, ebx2, inv;
    uint32_t eb_bits;
};

struct Geom {
    uint32_t T, B, D;  // T: tables of the whole payload (all destinations: ND * TD)
    uint32_t n;   // B*D symbols per table
    uint32_t G;   // groups per table
    uint32_t NG;  // T*G
    uint32_t ND;  // destinations: the payload is [ND][TD][B][D], every destination gets a container of its own
    uint32_t TD;  // tables per destination (= T of a container)
    uint32_t lz;  // 1: row matching (vector-based LZ step) is on for the tables flagged in Ws::rm_on
    uint32_t carry;  // 1: the codebook is carried from call to call (single-pass path)
    uint32_t sample;  // 1: the codebook comes from a sample of the payload (single-pass path, no state between calls)
    uint32_t S, R, K, LMAX;
    uint32_t dtype, es;
    uint32_t vec;  // 1: every table starts on a 16-byte (fp32) / 8-byte (fp16) boundary and n % 4 == 0
};

// per-table results of the codebook step
struct TMeta {
    uint32_t n_used, sym_lo, sym_hi, n_outliers;
};

// offsets of the sections of one container (one destination) whose position depends on the geometry alone
struct FixedLayout {
    uint64_t off_group, off_chunk, off_payload;
};

inline __host__ __device__ FixedLayout fixed_layout(const Geom& g) {
    FixedLayout F;
    const uint64_t ngd = (uint64_t)g.TD * g.G;  // groups of one container
    F.off_group = (kHeaderBytes + (uint64_t)kDirBytes * g.TD + 15ull) & ~15ull;
    F.off_chunk = (F.off_group + 4ull * ngd + 15ull) & ~15ull;
    F.off_payload = (F.off_chunk + (uint64_t)kW * ngd + 15ull) & ~15ull;
    return F;
}

// Single-pass path: a group's words (its chunks', then two per escape) wait in a slot of the workspace until the scan
// over the groups' totals has placed them.  A slot takes the worst case: every chunk full of the longest codes, every
// element an escape.
inline __host__ __device__ uint64_t carry_slot_words(const Geom& g) {
    return (uint64_t)kW * (((uint64_t)g.S * g.LMAX + 31ull) / 32ull) + 2ull * kW * g.S;
}

// DLC_FLAG_SAMPLE_CODEBOOK: the groups of a table whose symbols are counted for its codebook: groups 0, stride,
// 2 * stride, ..., `ns` of them: as many as hold kSampleElems elements, but no more than a quarter of the table's
// groups (rounded up), so that the sample of a small table is not the whole table
constexpr uint32_t kSampleElems = 65536;
inline __host__ __device__ void sample_groups(const Geom& g, uint32_t* ns, uint32_t* stride) {
    const uint32_t gs = kW * g.S;
    const uint32_t want = (kSampleElems + gs - 1u) / gs, quarter = (g.G + 3u) / 4u;
    *ns = want < quarter ? want : quarter;  // (at least one: G >= 1)
    *stride = g.G / *ns;                    // (>= 1: ns <= G)
}

constexpr uint32_t kPlaceGroups = 4;  // groups a work-group of k_post places: one per wavefront, many short wavefronts keep enough loads in flight
constexpr uint32_t kSumBlock = 32;   // groups whose totals are added up on the way (single-pass path)
inline __host__ __device__ uint32_t sum_blocks_per_dest(const Geom& g) { return (g.TD * g.G + kSumBlock - 1u) / kSumBlock; }

// small control block; `status` is sticky until read by the host, the rest is cleared per call
struct Ctrl {
    uint32_t ticket;  // ordered work-group ids of the encode kernel
    uint32_t abort;   // kAbort* bits: why (part of) the call's output is not valid
    uint32_t dest_done;  // destinations whose container the finalize kernel has finished (zero between calls)
    uint32_t pad1;
    int32_t status;   // first device-side error
    uint32_t collide; // statistics: a hash match whose rows differ
};

// Ctrl::abort: a container did not fit its capacity (the finalize kernel finds that out again for the container
// concerned: other destinations' containers stay valid); an internal wait ran out (nothing of the call is valid)
constexpr uint32_t kAbortCapacity = 1, kAbortInternal = 2;

struct DecTable {
    uint32_t valid, n_used, sym_lo, n_outliers;
    float ebx2;
    uint32_t pad;
    uint64_t ref_off;  // row matching: byte offset of the table's u32 ref[B] in its container, 0 = none
};

// ---- device helpers -----------------------------------------------------------------------------
#if defined(__HIPCC__)

__device__ __forceinline__ void set_status(Ctrl* c, int32_t code) { atomicCAS(&c->status, 0, code); }

// binary32 -> binary16, round to nearest even, of a value that is already a rounded binary32 number.  The value is
// pinned in a register first: handed a product directly, the compiler merges the multiply and the conversion into
// one mixed-precision instruction (v_fma_mixlo_f16), which rounds once, from the exact product, instead of twice,
// and that differs from "binary32 product, then binary16" whenever the binary32 product lands on a binary16 tie.
__device__ __forceinline__ __half half_rne(float v) {
    asm("" : "+v"(v));
    return __float2half_rn(v);
}

// Quantisation encoder without predictor: bin = rne(x / 2eb), taken as one binary32 multiply by the
// rounded reciprocal; escape (symbol 0) when the bin is outside (-R, R) or the reconstruction misses eb.
template <bool F16>
__device__ __forceinline__ uint32_t quant_symbol(float x, const QParam& q, float Rf, int R) {
    float r = __builtin_rintf(x * q.inv);
    float xh = r * q.ebx2;
    if constexpr (F16) xh = __half2float(half_rne(xh));
    float d = x - xh;
    bool ok = (__builtin_fabsf(r) < Rf) && (__builtin_fabsf(d) <= q.eb);
    return ok ? (uint32_t)((int)r + R) : 0u;
}

// Four consecutive elements of a group: `gbase` points at the group's first element (uniform over the
// wavefront), `off` is the element offset inside the group (off % 4 == 0, off < 64*S), `rem` the number of
// table elements from the group's start on.  Returns the mask of valid positions (off + v < rem); raw[]
// holds the bit patterns.  Branch-free: a position past the end reads the group's first element instead
// (always a legal address) and is masked out, so that the loads of several turns can be in flight together;
// offsets stay 32-bit so that one scalar base and one small vector offset address every load.
template <bool F16, bool VEC>
__device__ __forceinline__ uint32_t load4(const void* gbase, uint32_t off, uint32_t rem, float x[4], uint32_t raw[4]) {
    const char* gb = static_cast<const char*>(gbase);
    if constexpr (VEC) {
        const bool in = off < rem;
        const uint32_t o2 = in ? off : 0u;
        // streaming loads: the payload is read once per kernel and is larger than the caches, so it is kept from
        // displacing what the caches hold (measured: the histogram kernel 150 -> 88 us inside the compress/decompress loop)
        if constexpr (F16) {
            typedef uint32_t u2v __attribute__((ext_vector_type(2)));
            const u2v w = __builtin_nontemporal_load(reinterpret_cast<const u2v*>(gb + o2 * 2u));
            raw[0] = w.x & 0xFFFFu; raw[1] = w.x >> 16; raw[2] = w.y & 0xFFFFu; raw[3] = w.y >> 16;
#pragma unroll
            for (int v = 0; v < 4; ++v) x[v] = __half2float(__ushort_as_half((unsigned short)raw[v]));
        } else {
            typedef uint32_t u4v __attribute__((ext_vector_type(4)));
            const u4v w = __builtin_nontemporal_load(reinterpret_cast<const u4v*>(gb + o2 * 4u));
            raw[0] = w.x; raw[1] = w.y; raw[2] = w.z; raw[3] = w.w;
#pragma unroll
            for (int v = 0; v < 4; ++v) x[v] = __uint_as_float(raw[v]);
        }
        return in ? 0xFu : 0u;
    } else {
        uint32_t m = 0;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const bool in = off + v < rem;
            const uint32_t o2 = in ? off + v : 0u;
            m |= in ? (1u << v) : 0u;
            if constexpr (F16) {
                raw[v] = __builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(gb + o2 * 2u));
                x[v] = __half2float(__ushort_as_half((unsigned short)raw[v]));
            } else {
                raw[v] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(gb + o2 * 4u));
                x[v] = __uint_as_float(raw[v]);
            }
        }
        return m;
    }
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, uint32_t lane) {
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t u = __shfl_up(v, o, 64);
        if (lane >= (uint32_t)o) v += u;
    }
    return v;
}

// Exclusive prefix sum over a work-group of NW wavefronts (blockDim.x == 64*NW); every thread gets the
// grand total in *total.  `red` is NW+1 words of LDS.  Two barriers.
template <int NW>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* red, uint32_t tid, uint32_t* total) {
    const uint32_t lane = tid & 63u, wave = tid >> 6;
    const uint32_t incl = wave_incl_scan(v, lane);
    if (lane == 63) red[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const uint32_t w = lane < (uint32_t)NW ? red[lane] : 0u;
        const uint32_t wi = wave_incl_scan(w, lane);
        if (lane < (uint32_t)NW) red[lane] = wi - w;
        if (lane == NW - 1) red[NW] = wi;
    }
    __syncthreads();
    const uint32_t r = red[wave] + incl - v;
    *total = red[NW];
    return r;
}

#endif  // __HIPCC__

// ---- kernel launchers (defined next to their kernels) --------------------------------------------
struct Ws;  // workspace, see dlc_api.hip

hipError_t launch_quantize(const Geom& g, const void* payload, const QParam* qp, uint16_t* sym, hipStream_t s);
hipError_t launch_compress(const Geom& g, const void* payload, uint8_t* out, uint64_t capacity, uint64_t* out_bytes,
                           const Ws& w, uint64_t epoch, bool carry_ready, int prof_level, void* prof, hipStream_t s);
hipError_t launch_row_match(const Geom& g, const void* payload, const Ws& w, hipStream_t s);
// the row hash's multipliers, eight words per 4-byte piece of a row (six used), computed on the host once
void row_match_multipliers(uint32_t* mult, uint32_t n_pieces);
hipError_t row_match_set_attributes();
// per table and set: own[row] = the smallest row index whose hash equals the row's (see k_rm_sets)
hipError_t launch_row_sets(const Geom& g, uint32_t n_sets, const uint8_t* on, const uint64_t* rowhash, uint32_t* own,
                           uint32_t* unique, Ctrl* ctrl, hipStream_t s);
hipError_t launch_decompress(const Geom& g, const uint8_t* comp, uint64_t comp_bytes, void* out, const Ws& w,
                             int prof_level, void* prof, hipStream_t s);
hipError_t launch_stats(const Geom& g, const void* payload, const QParam* probe, const Ws& w, uint32_t salt,
                        hipStream_t s);

// device workspace of a context
struct Ws {
    uint8_t* base = nullptr;
    size_t bytes = 0;
    // compress
    QParam* qp = nullptr;          // [T]
    uint32_t* hist = nullptr;      // [T][K] zero between calls
    uint32_t* hist_view = nullptr; // [T][K] copy of the last call's histogram (inspection)
    Ctrl* ctrl = nullptr;          // ticket and abort are zero between calls
    TMeta* tmeta = nullptr;        // [T]
    uint16_t* enc = nullptr;       // [T][K]  len << 12 | codeword
    uint8_t* lens = nullptr;       // [T][K]
    uint64_t* state = nullptr;     // [NG] look-back records
    uint32_t* word_start = nullptr;  // [T]
    uint32_t* word_end = nullptr;    // [T]
    uint8_t* sym_plane = nullptr;  // [T][G*64*S] window index of every element (255: see the element itself)
    uint32_t* esc_count = nullptr; // [T] escapes of the call (single-pass path); zero between calls
    // row matching (allocated only with DLC_FLAG_ROW_MATCH)
    uint8_t* rm_on = nullptr;      // [T] 1: the table's repeated rows are stored as references
    uint32_t* rm_ref = nullptr;    // [T][B] first row of the batch with the row's content (the row itself: a coded row)
    uint64_t* rm_hash = nullptr;   // [T][B] row hashes
    uint32_t* rm_own = nullptr;    // [T][B] the smallest row index with the row's hash
    uint32_t* rm_mult = nullptr;   // [D/4][8] multipliers of the row hash
    uint32_t carry = 0;            // 1: the codebook is carried from call to call (single-pass path)
    uint32_t sample = 0;           // 1: the codebook comes from a sample of the payload (single-pass path)
    uint32_t* slots = nullptr;     // [NG][carry_slot_words] the groups' words before they are placed (single-pass path)
    uint32_t* gtot = nullptr;      // [NG] words of every group (single-pass path)
    uint16_t* enc_next = nullptr;  // single-pass path: the codebook for the next call is built while this call's is still
    uint8_t* lens_next = nullptr;  // being read; the two sets change places after every call
    TMeta* tmeta_next = nullptr;
    uint32_t* bsum = nullptr;      // [ND][ceil(TD*G / kSumBlock)] words of every block of groups (this call's)
    uint32_t* bsum_next = nullptr; // the next call's, cleared while this call's are read; the two change places after every call
    // decompress
    DecTable* dtab = nullptr;      // [T] row matching: what the reference check found
    uint32_t* dec_esc = nullptr;   // [T] escapes the decode kernel has applied; zero between calls
    uint32_t* dec_arrive = nullptr;  // [T] work-groups of the decode kernel that are done with the table; zero between calls
    // statistics (allocated on first use)
    uint8_t* stats_base = nullptr;
    size_t stats_bytes = 0;
    QParam* probe = nullptr;       // [T]
    uint64_t* rowhash = nullptr;   // [2][T][B] row hashes: raw bits, symbols at the probe bound
    uint32_t* st_own = nullptr;    // [2][T][B] the smallest row index with the row's hash
    uint32_t* st_mult = nullptr;   // [D][4] multipliers of the row hashes
    uint32_t* st_minmax = nullptr; // [T][2] order-preserving encodings
    uint32_t* st_unique = nullptr; // [T][2]
};

// profiling hooks used by the launchers (implemented in dlc_api.hip)
void prof_begin(void* prof, int slot, hipStream_t s);
void prof_end(void* prof, int slot, hipStream_t s);
enum ProfSlot { P_HIST = 0, P_CODEBOOK, P_ENCODE, P_FINALIZE, P_DECODE, P_CARRY, P_POST, P_NSLOTS };
inline bool prof_on(int level, int slot) {
    return level >= 2 || (level == 1 && (slot == P_ENCODE || slot == P_DECODE || slot == P_CARRY));
}

}  // namespace dlc
