// Single-pass compression with a codebook that exists before the payload is read, for one chunk size S (DLC_S,
// defined by the including source file): the codebook carried over from the previous call (below), or the one built
// from a sample of this call's payload just before (DLC_FLAG_SAMPLE_CODEBOOK: same kernel, same rules, no counting).
//
// The symbol distribution of a table changes little from one training iteration to the next (Section IV-C of the
// paper: the value distributions stay put through the phases of training), so the codebook built from the previous
// call's payload can code this call's.  That removes the histogram -> codebook -> encode dependency: the payload is
// read from memory once, and the histogram of this call is counted on the way, for the next call's codebook.
//   - a symbol the carried codebook has no code for becomes an escape (symbol 0 plus a record with the raw
//     value), so the error bound holds whatever the new payload looks like; the carried codebook always has a
//     code for symbol 0 (its count is raised by one when the codebook is built)
//   - the container is the same as that of the two-pass path; the decoder cannot tell them apart
//
// The kernel is bound by what a wavefront issues per element, so the walk is built to issue little:
//   - the quantiser's bin goes straight from the float pipeline to an LDS address (one fused multiply-add, a clamp, a
//     conversion): the address of the bin's word in this lane's copy of the code table, which holds codeword and
//     length in its low half and the bin's count in its high half, so one address serves the look-up and the count
//     (an atomic add of 1 << 16); neighbouring bins lie in neighbouring LDS banks
//   - the bound test of the quantiser is first taken with a fused multiply-add and a bound that is a little
//     tighter; only an element that fails this (one in a few thousand) is tested again with the quantiser's own
//     two roundings, so the decision is the quantiser's, bit for bit
//   - four codewords are joined and appended at once when they have at most 32 bits together (the rule), and the
//     word they complete is written to LDS without a branch: the store goes to the row of the last complete word,
//     again and again until a new one is complete
// ------------------------------------------------------------------------------------------------
#include "dlc_codec_dev.h"

#define DLC_CAT2(a, b) a##b
#define DLC_CAT(a, b) DLC_CAT2(a, b)

namespace dlc {

typedef __attribute__((address_space(3))) uint32_t lds_u32;

constexpr uint32_t kCarryBlk = 2;   // units (16-byte loads per lane) worked on together
constexpr uint32_t kCarryLoad = 2;  // units loaded together, one such block ahead of the work (4: registers spill, slower)

// The kernel's code table: row i in [1, 255] stands for symbol win_lo + i - 1; rows 0 and 256 for everything else
// (a symbol outside the window, NaN, a position past the end of the table).  A row is one word: codeword in bits 0-11,
// length in bits 12-15 (0: the carried codebook has no code for the symbol, or the row is 0 or 256), the row's count
// in bits 16-31.  A copy of the table serves a quarter of a work-group's 65536 elements, so a count fits its 16 bits.
constexpr uint32_t kCarryRows = 257;
constexpr uint32_t kCarryRowBytes = 4;
constexpr uint32_t kCarryCopies = 4;   // copies of the table (copy = lane mod kCarryCopies): spreads the counts of a popular bin
constexpr uint32_t kCarryCopyBytes = (kCarryRows + 7u) * kCarryRowBytes;  // a copy starts eight banks after the one before
static_assert(kCarryCopies * 65536u > 4u * 64u * 256u && 4u * 64u * 256u / kCarryCopies < 65536u, "a count must fit 16 bits");
constexpr uint32_t kCarryRecs = 128;  // escapes a wavefront remembers in LDS (offsets in the group); a group with more walks its elements again

// LDS staging of a wavefront, [row][lane]: row 0 takes the stores made before a chunk's first word is complete, row
// k + 1 holds word k of the lane's chunk, the last row takes what does not fit (a group with such a chunk is walked
// again, straight to memory)
__host__ __device__ constexpr uint32_t carry_stage_words(uint32_t cap) { return (cap + 2u) * kW; }

// A SIMD serves the oldest of its wavefronts first, so of the four work-groups that share a compute unit the one
// launched first runs ahead and the last one trails (lifetimes 89, 93, 98, 103 us by launch order on an MI355X), and
// the kernel lasts as long as the slowest.  Wave priorities that rotate through the four work-groups, a step every
// four turns of the walk, give each of them every place in the queue for a quarter of the time: they then finish
// within 3 us of each other instead of 13, and the kernel is 5 us shorter.
__device__ __forceinline__ void set_wave_priority(uint32_t p) {  // (the instruction takes its operand as an immediate)
    switch (p & 3u) {
        case 0: __builtin_amdgcn_s_setprio(0); break;
        case 1: __builtin_amdgcn_s_setprio(1); break;
        case 2: __builtin_amdgcn_s_setprio(2); break;
        default: __builtin_amdgcn_s_setprio(3); break;
    }
}

struct CarryEnv {
    const uint8_t* gbase;  // first element of the group
    uint32_t rem;          // elements of the table from there on
    uint32_t lane;
    QParam q;
    float eb_sure;         // a bound a little below q.eb: an element inside it is inside q.eb whichever way it is rounded
    float Rf;
    int R;
    float bias;            // LDS address of this lane's row of bin 0, as a float
    float lo, hi;          // LDS addresses of this lane's rows 0 and 256, as floats
    uint32_t row0;         // the same as an integer
    uint32_t win_lo;
    const uint16_t* enc_t;
    uint32_t* hist_t;
    uint32_t gstart;       // index of the group's first element in the table
    uint16_t* recs;        // LDS: where in the group the wavefront has met escapes, kCarryRecs at most
    uint32_t sp_base;      // LDS address of this lane's column of the staging rows
    uint32_t row_max;      // the last staging row
    uint32_t* dst;         // second walk of a group that did not fit its staging rows: the lane's chunk in memory
    uint32_t rank;         // which of the work-groups sharing a compute unit this one is, by launch order (0..3)
    uint32_t count;        // 0: nobody wants this call's counts (the codebook is not carried to the next call)
};

struct CarryState {
    uint64_t acc;   // the chunk's bits so far, the latest at the low end
    uint32_t nbt;   // how many
    uint32_t esc;   // escapes of this lane
    uint32_t nrec;  // escapes of the wavefront so far (uniform)
};

// the word the chunk's bits have completed last goes to its staging row (row 0 while there is none)
__device__ __forceinline__ void carry_flush(const CarryEnv& E, const CarryState& S) {
    const uint32_t row = min(S.nbt >> 5, E.row_max);
    const uint32_t word = __builtin_amdgcn_alignbit((uint32_t)(S.acc >> 32), (uint32_t)S.acc, S.nbt);  // (shift: nbt mod 32)
    *reinterpret_cast<lds_u32*>(E.sp_base + row * (kW * 4u)) = word;
}

// the same for a walk that writes a chunk straight to memory (the chunks' places are known by then): a word goes
// out once, when it is complete (S.nrec counts the words written: the second walk keeps no records)
__device__ __forceinline__ void carry_flush_mem(const CarryEnv& E, CarryState& S) {
    const uint32_t k = S.nbt >> 5;
    if (k != S.nrec) {
        E.dst[k - 1u] = __builtin_amdgcn_alignbit((uint32_t)(S.acc >> 32), (uint32_t)S.acc, S.nbt);
        S.nrec = k;
    }
}

// codeword and length of an element the table had no answer for, with the quantiser's own arithmetic: a symbol
// outside the window or without a code in the carried codebook, an escape, a position past the end of the table.
// Puts the count right where the walk's count (on row `a` of the table) was not the symbol's.
template <bool F16>
__device__ __forceinline__ void carry_slow_entry(const CarryEnv& E, float x, bool valid, uint32_t a, uint32_t& len,
                                                 uint32_t& code, bool& is_esc, bool count) {
    is_esc = false;
    if (!valid) { len = 0; code = 0; return; }
    const uint32_t c = quant_symbol<F16>(x, E.q, E.Rf, E.R);
    if (count) {
        const uint32_t row = (a - E.row0) / kCarryRowBytes;
        const uint32_t rowsym = (row >= 1u && row <= kCarryRows - 2u) ? E.win_lo + row - 1u : 0xFFFFFFFFu;
        if (c != rowsym) {
            if (rowsym != 0xFFFFFFFFu)  // (an escape whose bin lies in the window was counted there)
                __hip_atomic_fetch_sub(reinterpret_cast<lds_u32*>(a), 0x10000u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            atomicAdd(&E.hist_t[c], 1u);
        }
    }
    uint32_t ent = E.enc_t[c];
    if (c == 0u || (ent >> 12) == 0u) {
        ent = E.enc_t[0];
        is_esc = true;
    }
    len = ent >> 12;
    code = ent & 0xFFFu;
}

// One block of kCarryBlk units already loaded: quantise, count, look up, append.
// REWALK: the group is walked a second time because a chunk did not fit its staging rows; nothing is counted or
// recorded again, and the words go to memory.
template <bool F16, bool FULL, bool REWALK>
__device__ __forceinline__ void carry_block(const CarryEnv& E, const float (&x)[kCarryBlk][4], const uint32_t (&valid)[kCarryBlk],
                                            uint32_t jb, CarryState& S) {
    uint32_t a[kCarryBlk][4];
    bool sure = true;  // every element of the block passed the tighter bound test (a lane mask)
#pragma unroll
    for (uint32_t u = 0; u < kCarryBlk; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float xv = x[u][v];
            const float r = __builtin_rintf(xv * E.q.inv);
            if constexpr (F16) {  // (the reconstruction is rounded to half: the quantiser's own test, as it is)
                const float xh = __half2float(half_rne(r * E.q.ebx2));
                sure = sure & (__builtin_fabsf(xv - xh) <= E.q.eb);
            } else {
                sure = sure & (__builtin_fabsf(__builtin_fmaf(-r, E.q.ebx2, xv)) <= E.eb_sure);
            }
            // exact: small integers (a bin far outside the window is clamped whatever its rounding)
            const float t = __builtin_amdgcn_fmed3f(__builtin_fmaf(r, (float)kCarryRowBytes, E.bias), E.lo, E.hi);
            a[u][v] = (uint32_t)t;
            if constexpr (!FULL) {
                if (!((valid[u] >> v) & 1u)) a[u][v] = E.row0;
            }
        }
    // all look-ups, then all counts: the look-ups must not queue behind the (slower) atomic updates, whose results
    // nobody waits for
    uint32_t len[kCarryBlk][4], code[kCarryBlk][4];
#pragma unroll
    for (uint32_t u = 0; u < kCarryBlk; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) code[u][v] = *reinterpret_cast<lds_u32*>(a[u][v]);
    if (!REWALK && E.count != 0u) {  // (uniform: with a sampled codebook nobody reads the counts, and the walk is 4 us shorter without them)
#pragma unroll
        for (uint32_t u = 0; u < kCarryBlk; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                __hip_atomic_fetch_add(reinterpret_cast<lds_u32*>(a[u][v]), 0x10000u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
#pragma unroll
    for (uint32_t u = 0; u < kCarryBlk; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            len[u][v] = (code[u][v] >> 12) & 15u;
            code[u][v] &= 0xFFFu;
        }
    if (__ballot(!sure) != 0ull) {
        // one block in ten or so: the bound test again, with the quantiser's own two roundings; an element that fails
        // it has no answer in the table (it is an escape) and goes the long way below
#pragma unroll
        for (uint32_t u = 0; u < kCarryBlk; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float xv = x[u][v];
                float xh = __builtin_rintf(xv * E.q.inv) * E.q.ebx2;
                if constexpr (F16) xh = __half2float(half_rne(xh));
                len[u][v] = (__builtin_fabsf(xv - xh) <= E.q.eb) ? len[u][v] : 0u;
            }
    }
#pragma unroll
    for (uint32_t u = 0; u < kCarryBlk; ++u) {
        if (__ballot(min(min(len[u][0], len[u][1]), min(len[u][2], len[u][3])) == 0u) != 0ull) {
            // rare: an element without an answer from the table (length 0)
            uint32_t em = 0;  // which of the four are escapes
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (len[u][v] != 0u) continue;
                bool is_esc;
                carry_slow_entry<F16>(E, x[u][v], FULL || ((valid[u] >> v) & 1u), a[u][v], len[u][v], code[u][v], is_esc, !REWALK && E.count != 0u);
                if (is_esc && !REWALK) { ++S.esc; em |= 1u << v; }
            }
            // the records of these escapes, in element order (the walk meets the elements of a group in
            // increasing index: turn, lane, position); their offsets are kept while they fit.
            if (__ballot(em != 0u) != 0ull) {
                const uint32_t cnt = __popc(em);
                const uint32_t incl = wave_incl_scan(cnt, E.lane);
                uint32_t r = S.nrec + incl - cnt;
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if ((em >> v) & 1u) {
                        if (r < kCarryRecs) E.recs[r] = (uint16_t)(E.lane * kV + (jb + u) * (kW * kV) + (uint32_t)v);
                        ++r;
                    }
                S.nrec += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            }
        }
        const uint32_t l01 = len[u][0] + len[u][1], l23 = len[u][2] + len[u][3], L = l01 + l23;
        const uint32_t c01 = (code[u][0] << len[u][1]) | code[u][1], c23 = (code[u][2] << len[u][3]) | code[u][3];
        if (__ballot(L > 32u) == 0ull) {
            // the rule: the four codewords as one piece of at most 32 bits
            S.acc = (S.acc << L) | ((c01 << l23) | c23);
            S.nbt += L;
            if constexpr (REWALK) carry_flush_mem(E, S); else carry_flush(E, S);
        } else {
            // two pieces of at most 24 bits
            S.acc = (S.acc << l01) | c01;
            S.nbt += l01;
            if constexpr (REWALK) carry_flush_mem(E, S); else carry_flush(E, S);
            S.acc = (S.acc << l23) | c23;
            S.nbt += l23;
            if constexpr (REWALK) carry_flush_mem(E, S); else carry_flush(E, S);
        }
    }
}

template <bool F16, bool VEC, bool FULL>
__device__ __forceinline__ void carry_load(const CarryEnv& E, uint32_t jb, float (&x)[kCarryLoad][4], uint32_t (&valid)[kCarryLoad]) {
    uint32_t raw[4];
#pragma unroll
    for (uint32_t u = 0; u < kCarryLoad; ++u)
        valid[u] = load4<F16, VEC>(E.gbase, E.lane * kV + (jb + u) * (kW * kV), FULL ? 0xFFFFFFFFu : E.rem, x[u], raw);
}

// One walk over a group: lane l codes chunk l (at turn j the four elements group_base + j*256 + 4*l .. +3).  The
// loads of the next kCarryLoad turns are issued before the current ones are worked on; those of the first turns
// (xa, va) are already on their way when the walk starts.
template <int S, bool F16, bool VEC, bool FULL, bool REWALK = false>
__device__ __forceinline__ void carry_walk(const CarryEnv& E, CarryState& St, float (&xa)[kCarryLoad][4], uint32_t (&va)[kCarryLoad]) {
    constexpr uint32_t N = (uint32_t)S / kV;  // turns
    static_assert(N % (2 * kCarryLoad) == 0 && kCarryLoad % kCarryBlk == 0, "two load blocks per trip, whole work blocks per load block");
    typedef const float (&XBlk)[kCarryBlk][4];
    typedef const uint32_t (&VBlk)[kCarryBlk];
    float xb[kCarryLoad][4];
    uint32_t vb[kCarryLoad];
    for (uint32_t jb = 0; jb < N; jb += 2 * kCarryLoad) {
        set_wave_priority(jb / (2 * kCarryLoad) + E.rank);
        carry_load<F16, VEC, FULL>(E, jb + kCarryLoad, xb, vb);
#pragma unroll
        for (uint32_t k = 0; k < kCarryLoad; k += kCarryBlk)
            carry_block<F16, FULL, REWALK>(E, reinterpret_cast<XBlk>(xa[k]), reinterpret_cast<VBlk>(va[k]), jb + k, St);
        if (jb + 2 * kCarryLoad < N) carry_load<F16, VEC, FULL>(E, jb + 2 * kCarryLoad, xa, va);
#pragma unroll
        for (uint32_t k = 0; k < kCarryLoad; k += kCarryBlk)
            carry_block<F16, FULL, REWALK>(E, reinterpret_cast<XBlk>(xb[k]), reinterpret_cast<VBlk>(vb[k]), jb + kCarryLoad + k, St);
    }
}

// escape records of one group under a carried codebook: as emit_escapes, but a symbol without a code is one too
template <int S, bool F16, bool VEC>
__device__ __forceinline__ void carry_emit_escapes(uint32_t* rec, uint32_t lane, const uint8_t* gbase, uint32_t gstart,
                                                   uint32_t rem, const QParam& q, float Rf, int R, const uint16_t* enc_t) {
    uint32_t opos = 0;
    for (uint32_t j = 0; j < (uint32_t)S / kV; ++j) {
        const uint32_t off = lane * kV + j * (kW * kV);
        float x[4];
        uint32_t raw[4];
        const uint32_t valid = load4<F16, VEC>(gbase, off, rem, x, raw);
        uint32_t esc = 0;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (!((valid >> v) & 1u)) continue;
            const uint32_t c = quant_symbol<F16>(x[v], q, Rf, R);
            if (c == 0u || (enc_t[c] >> 12) == 0u) esc |= 1u << v;
        }
        if (__ballot(esc != 0u) == 0ull) continue;
        const uint32_t cnt = __popc(esc);
        const uint32_t incl = wave_incl_scan(cnt, lane);
        uint32_t r = opos + incl - cnt;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if ((esc >> v) & 1u) {
                rec[2u * r] = gstart + off + v;
                rec[2u * r + 1] = raw[v];
                ++r;
            }
        opos += __shfl(incl, 63, 64);
    }
}

// A work-group takes `ipw` consecutive items (an item: four consecutive groups of one table, one per wavefront) and
// no work-group waits for another: a group's words go to the group's slot of the workspace, and the kernel that
// follows (k_post) puts them where the sums of the groups' totals say.  The grid is sized to what the chip holds at
// once, so the set-up of a work-group is paid once, the code table stays in LDS while the items are of one table,
// and the first loads of an item are on their way while the item before it is being written out.
template <int S, bool F16, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void k_encode_carry(const void* payload, Geom g, FixedLayout F, const QParam* qp,
                                                      const uint16_t* enc, uint8_t* out, uint64_t capacity, uint32_t bpt,
                                                      uint32_t* hist, uint32_t* esc_count, uint32_t* slots, uint64_t slot_words,
                                                      uint32_t* gtot, uint32_t* bsum, uint32_t ipw, uint32_t n_items, uint32_t count) {
    constexpr uint32_t CAP = (uint32_t)S / 8u;          // words of LDS per chunk: room for 4 bits per symbol
    constexpr uint32_t kStageWords = carry_stage_words(CAP);  // per wavefront
    constexpr uint32_t kGroupEls = kW * (uint32_t)S;
    __shared__ __align__(16) uint32_t s_tab[kCarryCopies * kCarryCopyBytes / 4u];
    __shared__ __align__(16) uint32_t s_stage[4 * kStageWords];
    __shared__ uint16_t s_recs[4 * kCarryRecs];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t win_lo = win_lo_of(g.R);
    uint32_t* const stage = s_stage + wave * kStageWords;
    const uint32_t i0 = blockIdx.x * ipw, i1 = min(n_items, i0 + ipw);
    // bpt == 0: tables of few groups.  An item is then any four consecutive groups of the payload (table after table),
    // so that no wavefront idles where a table has fewer than four groups left; every wavefront keeps a code table of
    // its own (one copy instead of four shared ones) and looks after it alone, and the work-group never meets at a barrier.
    const bool pw = bpt == 0u;
    CarryEnv E;
    E.lane = lane;
    E.Rf = (float)g.R;
    E.R = (int)g.R;
    E.row0 = (uint32_t)(uintptr_t)s_tab + (pw ? wave : (lane & (kCarryCopies - 1u))) * kCarryCopyBytes;
    E.lo = (float)E.row0;
    E.hi = (float)(E.row0 + (kCarryRows - 1u) * kCarryRowBytes);
    E.bias = (float)(E.row0 + (g.R - win_lo + 1u) * kCarryRowBytes);
    E.win_lo = win_lo;
    E.recs = s_recs + wave * kCarryRecs;
    E.sp_base = (uint32_t)(uintptr_t)stage + lane * 4u;
    E.row_max = CAP + 1u;
    E.count = count;
    E.rank = min(3u, blockIdx.x / ((gridDim.x + 3u) / 4u));  // (the grid is four work-groups per compute unit, handed out in rounds)
    // which group of which table an item gives this wavefront (grp >= G: none)
    auto where = [&](uint32_t item, uint32_t& t, uint32_t& grp) {
        if (pw) {
            const uint32_t gi = item * 4u + wave;
            t = gi / g.G;
            grp = gi - t * g.G;
            if (t >= g.T) { t = g.T - 1u; grp = g.G; }
        } else {
            t = item / bpt;
            grp = (item % bpt) * 4u + wave;
        }
    };
    // where an item's group of this wavefront lies
    auto locate = [&](uint32_t item, const uint8_t*& gbase, uint32_t& rem) {
        uint32_t t, grp;
        where(item, t, grp);
        const uint32_t gstart = grp * kGroupEls;
        gbase = static_cast<const uint8_t*>(payload) + ((size_t)t * g.n + gstart) * g.es;
        rem = grp < g.G ? g.n - gstart : 0u;
    };
    // this call's histogram of a table, for the next call's codebook: the window rows (sum of the copies; everything
    // else went to memory directly); the counts start again at zero
    auto merge_counts = [&](uint32_t t) {
        if (tid < kCarryRows - 2u) {
            uint32_t s = 0;
            for (uint32_t c = 0; c < kCarryCopies; ++c) {
                uint32_t& w = s_tab[c * (kCarryCopyBytes / 4u) + tid + 1u];
                s += w >> 16;
                w &= 0xFFFFu;
            }
            const uint32_t sym = win_lo + tid;
            if (s && sym < g.K && count) atomicAdd(&hist[(size_t)t * g.K + sym], s);
        }
    };
    // the same for a wavefront's own table (tables of few groups)
    uint32_t* const tab_w = s_tab + wave * (kCarryCopyBytes / 4u);
    auto merge_counts_wave = [&](uint32_t t) {
        for (uint32_t r = lane; r < kCarryRows - 2u; r += 64) {
            const uint32_t w = tab_w[r + 1u];
            tab_w[r + 1u] = w & 0xFFFFu;
            const uint32_t sym = win_lo + r;
            if ((w >> 16) && sym < g.K && count) atomicAdd(&hist[(size_t)t * g.K + sym], w >> 16);
        }
    };
    // the first item's first elements are asked for before anything else: their way from memory is the longest
    float xa[kCarryLoad][4];
    uint32_t va[kCarryLoad];
    locate(i0, E.gbase, E.rem);
    if (E.rem != 0u) {
        if (E.rem >= kGroupEls) carry_load<F16, VEC, true>(E, 0, xa, va);
        else carry_load<F16, VEC, false>(E, 0, xa, va);
    }
    uint32_t cur_t = 0xFFFFFFFFu, since_merge = 0;
    for (uint32_t item = i0; item < i1; ++item) {
        uint32_t t, grp;
        where(item, t, grp);
        const bool active = grp < g.G;  // uniform over the wavefront; an idle wavefront only takes part in the barriers
        // the destination this table belongs to: its container starts `capacity` bytes after the previous one and
        // its groups are numbered from 0
        const uint32_t dst = t / g.TD, tl = t - dst * g.TD;
        const uint16_t* enc_t = enc + (size_t)t * g.K;
        if (pw) {  // the wavefront's own table
            if (active && t != cur_t) {
                if (cur_t != 0xFFFFFFFFu) merge_counts_wave(cur_t);
                for (uint32_t row = lane; row < kCarryRows; row += 64) {
                    const uint32_t c = win_lo + row - 1u;
                    tab_w[row] = (row >= 1u && row <= kCarryRows - 2u && c < g.K && c != 0u) ? enc_t[c] : 0u;
                }
                __builtin_amdgcn_wave_barrier();
                cur_t = t;
                since_merge = 0;
            } else if (active && since_merge == 3u) {
                merge_counts_wave(cur_t);
                __builtin_amdgcn_wave_barrier();
                since_merge = 0;
            }
        } else if (t != cur_t) {  // uniform over the work-group
            if (cur_t != 0xFFFFFFFFu) {
                __syncthreads();  // every wavefront has finished counting
                merge_counts(cur_t);
                __syncthreads();
            }
            // the code table: every row of every copy, counts zero (rows 0 and 256, the escape symbol and everything
            // without a code take the rare path)
            for (uint32_t k = tid; k < kCarryCopies * kCarryRows; k += 256) {
                const uint32_t row = k % kCarryRows;
                const uint32_t c = win_lo + row - 1u;
                const uint32_t e = (row >= 1u && row <= kCarryRows - 2u && c < g.K && c != 0u) ? enc_t[c] : 0u;
                s_tab[(k / kCarryRows) * (kCarryCopyBytes / 4u) + row] = e;  // (length 0: no code; count 0)
            }
            __syncthreads();
            cur_t = t;
            since_merge = 0;
        } else if (since_merge == 3u) {  // (a copy's count of a row has 16 bits: three items of 16384 elements a copy fit)
            __syncthreads();
            merge_counts(cur_t);
            __syncthreads();
            since_merge = 0;
        }
        ++since_merge;
        const uint32_t gid = tl * g.G + (active ? grp : 0u);  // group number inside the container
        const uint32_t gstart = grp * kGroupEls;
        locate(item, E.gbase, E.rem);
        E.q = qp[t];
        // |x - r * 2eb| as one fused operation differs from the quantiser's two roundings by at most 2^-24 of |r * 2eb|
        // (|r| < R inside the table) plus a rounding of the difference: well inside R * 2^-21 of the bound
        E.eb_sure = E.q.eb * (1.0f - (float)g.R * 0x1p-21f);
        E.enc_t = enc_t;
        E.hist_t = hist + (size_t)t * g.K;
        E.gstart = gstart;
        const uint8_t* const gbase = E.gbase;
        const uint32_t rem = E.rem;
        const bool full = rem >= kGroupEls;

        CarryState St;
        St.acc = 0; St.nbt = 0; St.esc = 0; St.nrec = 0;
        if (active) {
            if (full) carry_walk<S, F16, VEC, true>(E, St, xa, va);
            else carry_walk<S, F16, VEC, false>(E, St, xa, va);
            if (St.nbt & 31u)  // the chunk's last, partly filled word
                *reinterpret_cast<lds_u32*>(E.sp_base + min((St.nbt >> 5) + 1u, E.row_max) * (kW * 4u)) =
                    (uint32_t)St.acc << (32u - (St.nbt & 31u));
        }
        // the next item's first elements: on their way while this item is written out
        auto ask_for_next = [&]() {
            if (item + 1u < i1) {
                CarryEnv En = E;
                locate(item + 1u, En.gbase, En.rem);
                if (En.rem != 0u) {
                    if (En.rem >= kGroupEls) carry_load<F16, VEC, true>(En, 0, xa, va);
                    else carry_load<F16, VEC, false>(En, 0, xa, va);
                }
            }
        };
        ask_for_next();
        const uint32_t nw = (St.nbt + 31u) >> 5;
        const bool spilled = __ballot(nw > CAP) != 0ull;  // uniform: a chunk of this group did not fit its LDS words
        const uint32_t n_esc = active ? wave_sum(St.esc) : 0u;
        const uint32_t incl = wave_incl_scan(nw, lane);
        const uint32_t lane_off = incl - nw;
        const uint32_t chunk_total = __shfl(incl, 63, 64);
        const uint32_t total = chunk_total + 2u * n_esc;  // 0 for an idle wavefront

        // The group's words in output order: a lane takes its chunk's words out of its column into registers and puts
        // them where they go in a run of chunk_total words over the same LDS (the columns are in registers by then).
        if (active && !spilled) {
            uint32_t wb[CAP];
#pragma unroll
            for (uint32_t k = 0; k < CAP; ++k) wb[k] = *reinterpret_cast<lds_u32*>(E.sp_base + (k + 1u) * (kW * 4u));
            __builtin_amdgcn_wave_barrier();
            const uint32_t lin = (uint32_t)(uintptr_t)stage + lane_off * 4u;
#pragma unroll
            for (uint32_t k = 0; k < CAP; ++k)
                if (k < nw) *reinterpret_cast<lds_u32*>(lin + k * 4u) = wb[k];
            __builtin_amdgcn_wave_barrier();
        }
        if (active) {
            const uint32_t gg = t * g.G + grp;  // the group's number in the whole payload
            if (lane == 0) {
                gtot[gg] = total;
                atomicAdd(&bsum[dst * sum_blocks_per_dest(g) + gid / kSumBlock], total);  // (integer sums: the order does not matter)
                if (n_esc) atomicAdd(&esc_count[t], n_esc);
            }
            // (the sections the geometry fixes always fit: the host checks)
            (out + (uint64_t)dst * capacity)[F.off_chunk + (uint64_t)gid * kW + lane] = (uint8_t)nw;
            uint32_t* gw = slots + (size_t)gg * slot_words;
            if (!spilled) {
                for (uint32_t k = lane; k < chunk_total; k += 64) gw[k] = stage[k];
            } else {
                // A chunk of the group has more words than its staging rows: the group is walked again, the same way
                // but for the counts and the records, and every lane writes its chunk's words to memory as they get
                // complete (4 bytes a lane and 64 lines an instruction: the slow way out, for payloads that take more
                // than 4 bits per symbol).  The loads of the next item, already on their way, are asked for again.
                E.dst = gw + lane_off;
                CarryState Sr;
                Sr.acc = 0; Sr.nbt = 0; Sr.esc = 0; Sr.nrec = 0;
                if (full) {
                    carry_load<F16, VEC, true>(E, 0, xa, va);
                    carry_walk<S, F16, VEC, true, true>(E, Sr, xa, va);
                } else {
                    carry_load<F16, VEC, false>(E, 0, xa, va);
                    carry_walk<S, F16, VEC, false, true>(E, Sr, xa, va);
                }
                if (Sr.nbt & 31u) E.dst[Sr.nbt >> 5] = (uint32_t)Sr.acc << (32u - (Sr.nbt & 31u));
                ask_for_next();
            }
            if (n_esc != 0u) {  // uniform over the wavefront
                uint32_t* rec = gw + chunk_total;
                if (n_esc <= kCarryRecs) {  // the records were kept on the way
                    for (uint32_t k = lane; k < n_esc; k += 64) {  // (the raw bits come from the payload: the float in hand
                        const uint32_t off = E.recs[k];             //  need not convert back to the same half-precision bits)
                        rec[2u * k] = gstart + off;
                        if constexpr (F16) rec[2u * k + 1] = reinterpret_cast<const uint16_t*>(gbase)[off];
                        else rec[2u * k + 1] = reinterpret_cast<const uint32_t*>(gbase)[off];
                    }
                } else {
                    carry_emit_escapes<S, F16, VEC>(rec, lane, gbase, gstart, rem, E.q, E.Rf, (int)g.R, enc_t);
                }
            }
            __builtin_amdgcn_wave_barrier();  // (the staging rows and the records are written again by the next item)
        }
    }
    if (pw) {
        if (cur_t != 0xFFFFFFFFu) merge_counts_wave(cur_t);
        return;
    }
    __syncthreads();  // every wavefront of the work-group has finished counting
    if (cur_t != 0xFFFFFFFFu) merge_counts(cur_t);
}

// work-groups the chip holds at once (four per compute unit: LDS and registers are sized for that)
static inline uint32_t DLC_CAT(carry_resident_, DLC_S)() {
    static uint32_t n = 0;
    if (n == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        n = 4u * (uint32_t)cus;
    }
    return n;
}

void DLC_CAT(launch_encode_carry_, DLC_S)(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w,
                                          uint64_t epoch, uint8_t* out, uint64_t capacity, uint32_t bpt, hipStream_t s) {
    constexpr int S = DLC_S;
    // tables of few groups, not a multiple of four: items run through the groups of all tables (the kernel's bpt == 0).
    // Only where nothing is counted (a sampled codebook): a wavefront's own table is a single copy, and with a carried
    // codebook the counts of a popular bin then queue up behind each other (128 x 32 pieces of 256 x 128, two groups
    // each: 142 -> 110 us without counts, 148 -> 178 us with them).
    const bool pw = w.sample != 0 && (g.G & 3u) != 0u && g.G < 16u;
    if (pw) bpt = 0;
    const uint32_t n_items = pw ? (g.NG + 3u) / 4u : g.T * bpt;
    const uint32_t ipw = (n_items + DLC_CAT(carry_resident_, DLC_S)() - 1u) / DLC_CAT(carry_resident_, DLC_S)();
    dim3 grid((n_items + ipw - 1u) / ipw), block(256);
    const bool f16 = g.dtype == DLC_F16;
#define DLC_ENC(FF, V)                                                                                                 \
    hipLaunchKernelGGL((k_encode_carry<S, FF, V>), grid, block, 0, s, payload, g, F, w.qp, w.enc, out, capacity, bpt, w.hist, \
                       w.esc_count, w.slots, (uint64_t)carry_slot_words(g), w.gtot, w.bsum, ipw, n_items, w.sample != 0 ? 0u : 1u)
    if (f16) { if (g.vec) DLC_ENC(true, true); else DLC_ENC(true, false); }
    else { if (g.vec) DLC_ENC(false, true); else DLC_ENC(false, false); }
#undef DLC_ENC
}

}  // namespace dlc
