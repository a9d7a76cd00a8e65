// Single-pass compression with a carried codebook, for one chunk size S (DLC_S, defined by the including source
// file).
//
// The symbol distribution of a table changes little from one training iteration to the next (Section IV-C of the
// paper: the value distributions stay put through the phases of training), so the codebook built from the previous
// call's payload can code this call's.  That removes the histogram -> codebook -> encode dependency: the payload is
// read from memory once, and the histogram of this call is counted on the way, for the next call's codebook.
//   - a symbol the carried codebook has no code for becomes an escape (symbol 0 plus a record with the raw
//     value), so the error bound holds whatever the new payload looks like; the carried codebook always has a
//     code for symbol 0 (its count is raised by one when the codebook is built)
//   - the container is the same as that of the two-pass path; the decoder cannot tell them apart
#include "dlc_codec_dev.h"

#define DLC_CAT2(a, b) a##b
#define DLC_CAT(a, b) DLC_CAT2(a, b)

namespace dlc {

typedef __attribute__((address_space(3))) uint32_t lds_u32;

constexpr uint32_t kCarryBlk = 2;   // units (16-byte loads per lane) worked on together
constexpr uint32_t kCarryLoad = 4;  // units loaded together, one such block ahead of the work

// hooks for micro-benchmarks (a step switched off); the library has them all on
#ifndef DLC_CX_COUNT
#define DLC_CX_COUNT(addr) carry_count(addr)
#endif
#ifndef DLC_CX_LOOKUP
#define DLC_CX_LOOKUP(addr) (*reinterpret_cast<lds_u32*>(addr))
#endif
#ifndef DLC_CX_SAMPLE
#define DLC_CX_SAMPLE(u) true
#endif
#ifndef DLC_CX_PAIRS
#define DLC_CX_PAIRS 1
#endif
#ifndef DLC_CX_STAGE
#define DLC_CX_STAGE(addr, word) (*reinterpret_cast<lds_u32*>(addr) = (word))
#endif

// phase clocks of one wavefront, for micro-benchmarks only (compiled out of the library)
#ifdef DLC_CX_STAMPS
__device__ long long g_cstamp[16];
#define DLC_CX_T(i) do { const long long now_ = (long long)__builtin_readcyclecounter(); cx_t[i] += now_ - cx_last; cx_last = now_; } while (0)
#define DLC_CX_TDECL long long cx_t[8] = {0, 0, 0, 0, 0, 0, 0, 0}; long long cx_last = (long long)__builtin_readcyclecounter();
#define DLC_CX_TARGS , long long (&cx_t)[8], long long& cx_last
#define DLC_CX_TPASS , cx_t, cx_last
extern "C" void dlc_debug_cstamps(long long* out) { (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_cstamp), sizeof(g_cstamp)); }
#else
#define DLC_CX_T(i)
#define DLC_CX_TDECL
#define DLC_CX_TARGS
#define DLC_CX_TPASS
#endif

// inclusive running maximum over the 64 lanes, in the vector unit (no lane reads through LDS)
__device__ __forceinline__ uint32_t wave_incl_max(uint32_t v) {
    // shifts inside a row of 16 lanes (a lane without a source gets 0), then the last lane of a row to the rows after it
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false));  // row_shr:1
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false));  // row_shr:2
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false));  // row_shr:4
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false));  // row_shr:8
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false));  // row_bcast:15 -> rows 1 and 3
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false));  // row_bcast:31 -> rows 2 and 3
    return v;
}

__device__ __forceinline__ void carry_count(uint32_t addr) {
    __hip_atomic_fetch_add(reinterpret_cast<lds_u32*>(addr), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// The kernel's own window: table index i in [1, 255] stands for symbol win_lo + i - 1; 0 and 256 for everything else
// (an escape, a symbol outside the window, NaN, a position past the end of the table).  The index comes straight
// out of the float pipeline as a byte offset, 4*i, clamped to [0, 1024].
constexpr uint32_t kCarryRows = 257;
constexpr uint32_t kCarryRecs = 128;  // escapes a wavefront remembers in LDS (offsets in the group); a group with more walks its elements again
// copies of a histogram row in LDS (copy = lane mod kCarryCopies).  Few, and loads only four turns ahead: the
// kernel is sized (LDS 40 KiB, 128 registers) so that four work-groups share a CU, which counts for more here than
// cheaper atomics or deeper prefetch (measured: 16 copies and eight turns ahead at three work-groups, 160 us; this, 153 us)
constexpr uint32_t kCarryCopies = 4;

// LDS staging of a wavefront: word k of chunk l at [k*65 + l] (stride 65: the words of one chunk fall into
// different banks when the chunk is copied out), CAP rows plus one that takes what does not fit
__host__ __device__ constexpr uint32_t carry_stage_words(uint32_t cap) { return (cap + 1u) * 65u; }

struct CarryEnv {
    const uint8_t* gbase;  // first element of the group
    uint32_t rem;          // elements of the table from there on
    uint32_t lane;
    QParam q;
    float Rf;
    int R;
    float bias4;           // 4 * (window index of bin 0 + 1)
    uint32_t win_lo;
    uint32_t a_tab;        // LDS address of the code table
    uint32_t lanebase;     // LDS address of this lane's copy of histogram row 0
    const uint16_t* enc_t;
    uint32_t* hist_t;
    uint32_t gstart;       // index of the group's first element in the table
    uint16_t* recs;        // LDS: where in the group the wavefront has met escapes, kCarryRecs at most
};

// One block of kCarryBlk units already loaded: quantise, count, look up, append.
// FIRST: count the histogram and the escapes; words go to LDS at sp (a lane's column, running address, clamped to
//        sp_lim: the row that takes what does not fit).   else: words go to memory at dst.
template <bool F16, bool FULL, bool FIRST>
__device__ __forceinline__ void carry_block(const CarryEnv& E, const float (&x)[kCarryBlk][4], const uint32_t (&valid)[kCarryBlk],
                                            uint32_t jb, uint64_t& acc, uint32_t& nb, uint32_t& sp, uint32_t sp_lim,
                                            uint32_t*& dst, uint32_t& esc, uint32_t& nrec DLC_CX_TARGS) {
    // table offsets of the whole block, then all look-ups, then all counts: the look-ups must not queue behind
    // the (slower) atomic updates, whose results nobody waits for
    uint32_t ab[kCarryBlk][4], eb_[kCarryBlk][4];
    DLC_CX_T(0);
#pragma unroll
    for (uint32_t u = 0; u < kCarryBlk; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            // the quantiser (same arithmetic as quant_symbol); the range test is left to the table (a symbol outside
            // (0, 2R) has no entry), the bound test sends the element to the rare path
            const float xv = x[u][v];
            const float r = __builtin_rintf(xv * E.q.inv);
            float xh = r * E.q.ebx2;
            if constexpr (F16) xh = __half2float(half_rne(xh));
            const float d = xv - xh;
            const bool ok = __builtin_fabsf(d) <= E.q.eb;
            const float t = __builtin_amdgcn_fmed3f(__builtin_fmaf(r, 4.0f, E.bias4), 0.0f, 1024.0f);  // exact: small integers
            ab[u][v] = ok ? (uint32_t)t : 0u;
            if constexpr (!FULL) {
                if (!((valid[u] >> v) & 1u)) ab[u][v] = 0u;
            }
        }
    DLC_CX_T(1);
#pragma unroll
    for (uint32_t u = 0; u < kCarryBlk; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) eb_[u][v] = DLC_CX_LOOKUP(E.a_tab + ab[u][v]);  // len << 16 | codeword; 0: not in the table
    if constexpr (FIRST) {
#pragma unroll
        for (uint32_t u = 0; u < kCarryBlk; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (DLC_CX_SAMPLE(u) && (FULL || ((valid[u] >> v) & 1u))) DLC_CX_COUNT(ab[u][v] * kCarryCopies + E.lanebase);  // rows 0 and 256 are not used
    }
    DLC_CX_T(2);
#pragma unroll
    for (uint32_t u = 0; u < kCarryBlk; ++u) {
        uint32_t a[4], e[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) { a[v] = ab[u][v]; e[v] = eb_[u][v]; }
        // rare: an escape, a symbol outside the window, a symbol the carried codebook has no code for
        if (__ballot(min(min(e[0], e[1]), min(e[2], e[3])) == 0u) != 0ull) {
            uint32_t em = 0;  // which of the four are escapes
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (e[v] != 0u) continue;
                if constexpr (!FULL) {
                    if (!((valid[u] >> v) & 1u)) continue;
                }
                const uint32_t c = quant_symbol<F16>(x[u][v], E.q, E.Rf, E.R);  // the symbol itself
                if constexpr (FIRST) {
                    if (a[v] - 4u >= 4u * (kCarryRows - 2u)) atomicAdd(&E.hist_t[c], 1u);  // window symbols were counted above
                }
                uint32_t ent = E.enc_t[c];
                if (c == 0u || (ent >> 12) == 0u) {
                    ent = E.enc_t[0];
                    ++esc;
                    em |= 1u << v;
                }
                e[v] = ((ent >> 12) << 16) | (ent & 0xFFFu);
            }
            if constexpr (FIRST) {
                // the records of these escapes, in element order (the walk meets the elements of a group in
                // increasing index: turn, lane, position); their offsets are kept while they fit.
                const uint32_t cnt = __popc(em);
                const uint32_t incl = wave_incl_scan(cnt, E.lane);
                uint32_t r = nrec + incl - cnt;
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if ((em >> v) & 1u) {
                        if (r < kCarryRecs) E.recs[r] = (uint16_t)(E.lane * kV + (jb + u) * (kW * kV) + (uint32_t)v);
                        ++r;
                    }
                nrec += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            }
        }
#pragma unroll
        for (int h = 0; h < 2 * DLC_CX_PAIRS; ++h) {
            const uint32_t l0 = e[2 * h] >> 16, l1 = e[2 * h + 1] >> 16;
            const uint32_t len = l0 + l1;  // a pair: at most 24 bits
            acc = (acc << len) | (((e[2 * h] & 0xFFFFu) << l1) | (e[2 * h + 1] & 0xFFFFu));
            nb += len;
            if (nb >= 32u) {
                nb -= 32u;
                const uint32_t word = (uint32_t)(acc >> nb);
                if constexpr (FIRST) {
                    DLC_CX_STAGE(min(sp, sp_lim), word);
                    sp += 65u * 4u;
                } else {
                    *dst++ = word;
                }
            }
        }
    }
    DLC_CX_T(3);
}

template <bool F16, bool VEC, bool FULL>
__device__ __forceinline__ void carry_load(const CarryEnv& E, uint32_t jb, float (&x)[kCarryLoad][4], uint32_t (&valid)[kCarryLoad]) {
    uint32_t raw[4];
#pragma unroll
    for (uint32_t u = 0; u < kCarryLoad; ++u)
        valid[u] = load4<F16, VEC>(E.gbase, E.lane * kV + (jb + u) * (kW * kV), FULL ? 0xFFFFFFFFu : E.rem, x[u], raw);
}

// One walk over a group: lane l codes chunk l (at turn j the four elements group_base + j*256 + 4*l .. +3).  The
// loads of the next kCarryLoad turns are issued before the current ones are worked on.
template <int S, bool F16, bool VEC, bool FULL, bool FIRST>
__device__ __forceinline__ void carry_walk(const CarryEnv& E, uint64_t& acc, uint32_t& nb, uint32_t& sp, uint32_t sp_lim,
                                           uint32_t*& dst, uint32_t& esc, uint32_t& nrec DLC_CX_TARGS) {
    constexpr uint32_t N = (uint32_t)S / kV;  // turns
    static_assert(N % (2 * kCarryLoad) == 0 && kCarryLoad % kCarryBlk == 0, "two load blocks per trip, whole work blocks per load block");
    typedef const float (&XBlk)[kCarryBlk][4];
    typedef const uint32_t (&VBlk)[kCarryBlk];
    float xa[kCarryLoad][4], xb[kCarryLoad][4];
    uint32_t va[kCarryLoad], vb[kCarryLoad];
    carry_load<F16, VEC, FULL>(E, 0, xa, va);
    for (uint32_t jb = 0; jb < N; jb += 2 * kCarryLoad) {
        carry_load<F16, VEC, FULL>(E, jb + kCarryLoad, xb, vb);
#pragma unroll
        for (uint32_t k = 0; k < kCarryLoad; k += kCarryBlk)
            carry_block<F16, FULL, FIRST>(E, reinterpret_cast<XBlk>(xa[k]), reinterpret_cast<VBlk>(va[k]), jb + k, acc, nb, sp, sp_lim, dst, esc, nrec DLC_CX_TPASS);
        if (jb + 2 * kCarryLoad < N) carry_load<F16, VEC, FULL>(E, jb + 2 * kCarryLoad, xa, va);
#pragma unroll
        for (uint32_t k = 0; k < kCarryLoad; k += kCarryBlk)
            carry_block<F16, FULL, FIRST>(E, reinterpret_cast<XBlk>(xb[k]), reinterpret_cast<VBlk>(vb[k]), jb + kCarryLoad + k, acc, nb, sp, sp_lim, dst, esc, nrec DLC_CX_TPASS);
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

template <int S, bool F16, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void k_encode_carry(const void* payload, Geom g, FixedLayout F, const QParam* qp,
                                                      const uint16_t* enc, Ctrl* ctrl, uint64_t* state, uint64_t epoch,
                                                      uint8_t* out, uint64_t capacity, uint32_t bpt, uint32_t* word_start,
                                                      uint32_t* word_end, uint32_t* hist, uint32_t* esc_count) {
    constexpr uint32_t CAP = (uint32_t)S / 8u;          // words of LDS per chunk: room for 4 bits per symbol
    constexpr uint32_t kStageWords = carry_stage_words(CAP);  // per wavefront
    __shared__ __align__(16) uint32_t s_hist[(kCarryRows + 3u) * kCarryCopies];
    __shared__ __align__(16) uint32_t s_tab[kCarryRows + 3u];  // by table index: len << 16 | codeword; 0 = no code
    __shared__ __align__(16) uint32_t s_stage[4 * kStageWords];
    __shared__ uint16_t s_recs[4 * kCarryRecs];
    __shared__ uint32_t s_wg, s_tot[4], s_excl, s_dead;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid == 0) s_wg = atomicAdd(&ctrl->ticket, 1u);
    {
        uint4* z = reinterpret_cast<uint4*>(s_hist);
        for (uint32_t k = tid; k < (kCarryRows + 3u) * kCarryCopies / 4u; k += 256) z[k] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    const uint32_t wg = __builtin_amdgcn_readfirstlane(s_wg);
    const uint32_t t = wg / bpt, b = wg % bpt;
    // the destination this table belongs to: its container starts `capacity` bytes after the previous one, its
    // groups are numbered and its words are placed from 0, so the scan over work-groups starts anew at its first
    const uint32_t dst = t / g.TD, tl = t - dst * g.TD;
    const uint32_t dom0 = dst * g.TD * bpt;
    out += (uint64_t)dst * capacity;
    const uint32_t win_lo = win_lo_of(g.R);
    const uint16_t* enc_t = enc + (size_t)t * g.K;
    uint32_t* hist_t = hist + (size_t)t * g.K;
    {
        // table index tid + 1 (1 .. 256); the escape symbol and everything without a code take the rare path
        const uint32_t c = win_lo + tid;
        const uint32_t e = (tid < kCarryRows - 2u && c < g.K && c != 0u) ? enc_t[c] : 0u;
        s_tab[tid + 1u] = ((e >> 12) << 16) | (e & 0xFFFu);
        if (tid == 0) s_tab[0] = 0u;
    }
    __syncthreads();
    const uint32_t grp = b * 4 + wave;
    const bool active = grp < g.G;  // uniform over the wavefront; an idle wavefront only takes part in the barriers
    const uint32_t gid = tl * g.G + (active ? grp : 0u);  // group number inside the container
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t gstart = grp * (kW * (uint32_t)S);
    CarryEnv E;
    E.gbase = tab + (size_t)gstart * g.es;
    E.rem = active ? g.n - gstart : 0u;
    E.lane = lane;
    E.q = qp[t];
    E.Rf = (float)g.R;
    E.R = (int)g.R;
    E.bias4 = 4.0f * (float)(g.R - win_lo + 1u);
    E.win_lo = win_lo;
    E.a_tab = (uint32_t)(uintptr_t)s_tab;
    E.lanebase = (uint32_t)(uintptr_t)s_hist + (lane & (kCarryCopies - 1u)) * 4u;
    E.enc_t = enc_t;
    E.hist_t = hist_t;
    E.gstart = gstart;
    E.recs = s_recs + wave * kCarryRecs;
    const uint8_t* const gbase = E.gbase;
    const uint32_t rem = E.rem;
    const QParam q = E.q;
    const float Rf = E.Rf;
    const bool full = rem >= kW * (uint32_t)S;
    uint32_t* const stage = s_stage + wave * kStageWords;
    const uint32_t sp0 = (uint32_t)(uintptr_t)stage + lane * 4u;  // word 0 of this lane's chunk
    const uint32_t sp_lim = sp0 + CAP * 65u * 4u;

    uint64_t acc = 0;
    uint32_t nb = 0, sp = sp0, my_esc = 0, nrec = 0;
    uint32_t* nodst = nullptr;
    DLC_CX_TDECL
    if (active) {
        if (full) carry_walk<S, F16, VEC, true, true>(E, acc, nb, sp, sp_lim, nodst, my_esc, nrec DLC_CX_TPASS);
        else carry_walk<S, F16, VEC, false, true>(E, acc, nb, sp, sp_lim, nodst, my_esc, nrec DLC_CX_TPASS);
        if (nb) {  // the chunk's last, partly filled word
            *reinterpret_cast<lds_u32*>(min(sp, sp_lim)) = (uint32_t)(acc << (32u - nb));
            sp += 65u * 4u;
        }
    }
    DLC_CX_T(4);
    const uint32_t nw = (sp - sp0) / (65u * 4u);
    const bool spilled = __ballot(nw > CAP) != 0ull;  // uniform: a chunk of this group did not fit its LDS words
    const uint32_t n_esc = active ? wave_sum(my_esc) : 0u;
    const uint32_t incl = wave_incl_scan(nw, lane);
    const uint32_t lane_off = incl - nw;
    const uint32_t chunk_total = __shfl(incl, 63, 64);
    const uint32_t total = chunk_total + 2u * n_esc;  // 0 for an idle wavefront

    if (lane == 0) s_tot[wave] = total;
    __syncthreads();  // also: every wavefront of the work-group has finished counting
    const uint32_t wg_total = s_tot[0] + s_tot[1] + s_tot[2] + s_tot[3];
    // The look-back over the records of earlier work-groups (first wavefront) takes a while: a work-group waits for
    // the slowest of those that started before it.  Meanwhile every wavefront already fetches its group's words
    // from the LDS columns, in output order, into registers; once the offset is known they only need storing.
    //   word i of the group belongs to the last non-empty chunk that starts at or before i.  Segment by segment
    //   of 64 words: the chunks that start inside the segment put (start << 8 | chunk) at their start's place
    //   in a 64-word scratch, and a running maximum spreads it over the words that follow (what the scratch
    //   still holds from earlier segments is smaller than the value carried in, so it never needs clearing).
    LookBack L;
    lb_init(L, wg, dom0);
    if (wave == 0) lb_publish_aggregate(state, epoch, wg, wg_total, lane, dom0);
    uint32_t wb[CAP];
    if (active && !spilled) {
        uint32_t* const heads = stage + CAP * 65u;  // the row that takes what does not fit is free now (nothing spilled)
        heads[lane] = 0u;
        const uint32_t mine = (lane_off << 8) | lane;
        uint32_t carry = 0u;
#pragma unroll
        for (uint32_t seg = 0; seg < CAP; ++seg) {
            const uint32_t base = seg * 64u;
            wb[seg] = 0u;
            if (base < chunk_total) {  // uniform
                if (nw != 0u && lane_off - base < 64u) heads[lane_off - base] = mine;
                __builtin_amdgcn_wave_barrier();
                uint32_t v = max(heads[lane], carry);
                __builtin_amdgcn_wave_barrier();
                v = wave_incl_max(v);
                carry = (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
                const uint32_t c = v & 0xFFu, k = base + lane - (v >> 8);
                if (base + lane < chunk_total) wb[seg] = stage[k * 65u + c];
            }
            if (wave == 0 && !L.done && (seg % 4u) == 3u) {  // uniform: one look-back step per four segments
                if (L.pending) (void)lb_consume(L, epoch, lane);
                if (!L.done) lb_issue(L, state, epoch, lane);
            }
        }
    }
    if (wave == 0) {
        lb_finish(L, state, epoch, wg, wg_total, lane, ctrl);
        if (lane == 0) { s_excl = L.excl; s_dead = L.failed ? 1u : 0u; }
    }
    // this call's histogram, for the next call's codebook: the window rows (sum of the copies, skewed start so that
    // the threads of a wavefront read different banks); everything else went to memory directly
    if (tid < kCarryRows - 2u) {
        const uint32_t* row = s_hist + (tid + 1u) * kCarryCopies;
        uint32_t s = 0;
        for (uint32_t c = 0; c < kCarryCopies; ++c) s += row[(c + tid) & (kCarryCopies - 1u)];
        const uint32_t sym = win_lo + tid;
        if (s && sym < g.K) atomicAdd(&hist_t[sym], s);
    }
    __syncthreads();
    DLC_CX_T(5);
    bool dead = s_dead != 0u;  // nothing may be written to the container
    uint32_t excl = s_excl;
    for (uint32_t k = 0; k < wave; ++k) excl += s_tot[k];
    if (F.off_payload + 4ull * ((uint64_t)excl + total) > capacity) {
        if (active && !dead && lane == 0) { set_status(ctrl, DLC_ECAPACITY); atomicOr(&ctrl->abort, kAbortCapacity); }
        dead = true;
    }
    if (!active) return;
    if (lane == 0) {
        if (grp == 0) word_start[t] = excl;
        if (grp == g.G - 1) word_end[t] = excl + total;
        if (n_esc) atomicAdd(&esc_count[t], n_esc);
    }
    if (dead) return;
    out[F.off_chunk + (uint64_t)gid * kW + lane] = (uint8_t)nw;
    if (lane == 0) reinterpret_cast<uint32_t*>(out + F.off_group)[gid] = excl;
    uint32_t* gw = reinterpret_cast<uint32_t*>(out + F.off_payload) + excl;
    if (!spilled) {
#pragma unroll
        for (uint32_t seg = 0; seg < CAP; ++seg)
            if (seg * 64u + lane < chunk_total) gw[seg * 64u + lane] = wb[seg];
    } else {
        // walk again, straight to memory now that the chunk's place is known (the group's elements are read again)
        uint64_t acc2 = 0;
        uint32_t nb2 = 0, sp2 = sp0, esc2 = 0, nrec2 = 0;
        uint32_t* dst = gw + lane_off;
        if (full) carry_walk<S, F16, VEC, true, false>(E, acc2, nb2, sp2, sp_lim, dst, esc2, nrec2 DLC_CX_TPASS);
        else carry_walk<S, F16, VEC, false, false>(E, acc2, nb2, sp2, sp_lim, dst, esc2, nrec2 DLC_CX_TPASS);
        if (nb2) *dst = (uint32_t)(acc2 << (32u - nb2));
    }
#ifdef DLC_CX_STAMPS
    DLC_CX_T(6);
    if (wg == DLC_CX_STAMPS && tid == 0)
        for (int i = 0; i < 8; ++i) g_cstamp[i] = cx_t[i];
#endif
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
            carry_emit_escapes<S, F16, VEC>(rec, lane, gbase, gstart, rem, q, Rf, (int)g.R, enc_t);
        }
    }
}

void DLC_CAT(launch_encode_carry_, DLC_S)(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w,
                                          uint64_t epoch, uint8_t* out, uint64_t capacity, uint32_t bpt, hipStream_t s) {
    constexpr int S = DLC_S;
    dim3 grid(g.T * bpt), block(256);
    const bool f16 = g.dtype == DLC_F16;
#define DLC_ENC(FF, V)                                                                                                 \
    hipLaunchKernelGGL((k_encode_carry<S, FF, V>), grid, block, 0, s, payload, g, F, w.qp, w.enc, w.ctrl, w.state, epoch, \
                       out, capacity, bpt, w.word_start, w.word_end, w.hist, w.esc_count)
    if (f16) { if (g.vec) DLC_ENC(true, true); else DLC_ENC(true, false); }
    else { if (g.vec) DLC_ENC(false, true); else DLC_ENC(false, false); }
#undef DLC_ENC
}

#ifdef DLC_CX_STAMPS
extern "C" int dlc_debug_carry_occupancy() {
    int n = -1;
    (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void*>(k_encode_carry<DLC_S, false, true>), 256, 0);
    return n;
}
#endif

}  // namespace dlc
