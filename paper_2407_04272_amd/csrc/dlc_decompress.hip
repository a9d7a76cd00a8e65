// Decompression kernels for gfx950: container validation, decode tables and chunk-parallel decode in one kernel,
// escape scatter, row copies.
#include <algorithm>

#include "dlc_internal.h"

namespace dlc {

__device__ __forceinline__ uint64_t d_a16(uint64_t x) { return (x + 15ull) & ~15ull; }

// What a work-group learns from the container about the table it decodes.  Every range test is written without an
// addition on the untrusted side (an offset near 2^64 must fail the test, not wrap past it).
struct DecHead {
    bool ok;
    uint32_t n_used, sym_lo, sym_hi, n_esc;
    float ebx2;
    uint64_t cb;           // byte offset of the table's code lengths
    uint64_t ref_off;      // row matching: byte offset of the table's u32 ref[B], 0 = none
    uint64_t words_total;  // payload words of the container
    uint64_t n_esc_total;  // escapes of the container
};

// Header against the context's geometry, the table's directory entry against the header.  `comp` is the start of the
// container, `comp_bytes` the room it has; `tl` the table's place in the container.  The same for every thread.
__device__ __forceinline__ DecHead dec_validate(const Geom& g, const FixedLayout& F, const uint8_t* comp,
                                                uint64_t comp_bytes, uint32_t tl) {
    DecHead H;
    H.ok = false; H.n_used = 0; H.sym_lo = 0; H.sym_hi = 0; H.n_esc = 0; H.ebx2 = 0.f; H.cb = 0; H.ref_off = 0;
    H.words_total = 0; H.n_esc_total = 0;
    if (comp_bytes < F.off_payload) return H;  // header, directory, group and chunk tables: their size is the geometry's
    // header and directory entry are read together (no test between the loads), then looked at
    const uint32_t* h = reinterpret_cast<const uint32_t*>(comp);
    const uint64_t* q = reinterpret_cast<const uint64_t*>(comp);
    const uint8_t* d = comp + kHeaderBytes + (uint64_t)kDirBytes * tl;
    const uint32_t* d32 = reinterpret_cast<const uint32_t*>(d);
    const uint64_t* d64 = reinterpret_cast<const uint64_t*>(d + 24);
    uint32_t hw[12];
#pragma unroll
    for (int k = 0; k < 12; ++k) hw[k] = h[k];
    uint64_t hq[7];
#pragma unroll
    for (int k = 0; k < 7; ++k) hq[k] = q[HQ_NOUT + k];
    uint32_t dw[6];
#pragma unroll
    for (int k = 0; k < 6; ++k) dw[k] = d32[k];
    const uint64_t d_cb = d64[0], d_ref = d64[1];
    bool ok = hw[H_MAGIC] == kMagic && hw[H_VERSION] == kVersion && hw[H_DTYPE] == g.dtype && hw[H_T] == g.TD &&
              hw[H_B] == g.B && hw[H_D] == g.D && hw[H_R] == g.R && hw[H_S] == g.S && hw[H_LMAX] == g.LMAX &&
              hw[H_W] == kW && hw[H_V] == kV && hw[H_NG] == g.TD * g.G;
    H.n_esc_total = hq[HQ_NOUT - HQ_NOUT];
    H.words_total = hq[HQ_WORDS - HQ_NOUT];
    const uint64_t off_cb = hq[HQ_OFF_CB - HQ_NOUT], total = hq[HQ_TOTAL - HQ_NOUT];
    // (the code-length blocks are padded to four bytes and every table has one, so at least four bytes follow the
    // payload section: the decode kernel may read the word at the payload's end)
    ok = ok && total <= comp_bytes && hq[HQ_OFF_GROUP - HQ_NOUT] == F.off_group && hq[HQ_OFF_CHUNK - HQ_NOUT] == F.off_chunk &&
         hq[HQ_OFF_PAYLOAD - HQ_NOUT] == F.off_payload && H.words_total <= 0xFFFFFFFFull &&
         H.n_esc_total <= (uint64_t)g.n * g.TD;
    ok = ok && off_cb == d_a16(F.off_payload + 4ull * H.words_total) && total >= off_cb && total - off_cb >= 4ull;
    const float eb = __uint_as_float(dw[0]);
    H.n_used = dw[1]; H.sym_lo = dw[2]; H.sym_hi = dw[3]; H.n_esc = dw[4];
    H.cb = d_cb;
    H.ref_off = d_ref;
    H.ebx2 = eb * 2.0f;
    ok = ok && eb > 0.f && eb < __builtin_inff() && dw[5] == g.G && H.sym_lo <= H.sym_hi && H.sym_hi < g.K &&
         H.n_used >= 1 && H.n_used <= H.sym_hi - H.sym_lo + 1u && H.n_esc <= g.n;
    ok = ok && H.cb >= off_cb && H.cb <= total && (uint64_t)(H.sym_hi - H.sym_lo + 1u) <= total - H.cb;
    // row matching: references behind the code-length blocks (only a context made for it decodes them, and the
    // kernels want a lane's four elements in one row)
    if (H.ref_off != 0)
        ok = ok && g.lz != 0 && (g.D % 4u) == 0 && (H.ref_off % 4u) == 0 && H.ref_off >= off_cb && H.ref_off <= total &&
             4ull * g.B <= total - H.ref_off;
    H.ok = ok;
    return H;
}

// ------------------------------------------------------------------------------------------------
// Row matching only: one work-group per table checks that every reference points back, at a row that is coded,
// and leaves the verdict (and where the references are) for the row-copy kernel.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_dec_refs(Geom g, FixedLayout F, const uint8_t* comp, uint64_t comp_bytes,
                                                  DecTable* dtab, Ctrl* ctrl) {
    __shared__ uint32_t s_ok;
    const uint32_t tid = threadIdx.x, t = blockIdx.x;
    const uint32_t dst = t / g.TD, tl = t - dst * g.TD;
    comp += (uint64_t)dst * comp_bytes;
    const DecHead H = dec_validate(g, F, comp, comp_bytes, tl);
    if (tid == 0) s_ok = H.ok ? 1u : 0u;
    __syncthreads();
    if (H.ok && H.ref_off != 0) {
        const uint32_t* ref = reinterpret_cast<const uint32_t*>(comp + H.ref_off);
        for (uint32_t r0 = tid; r0 < g.B; r0 += 256u * 4u) {  // four rows in flight per thread
            uint32_t o[4], oo[4];
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                const uint32_t r = r0 + k * 256u;
                o[k] = r < g.B ? ref[r] : 0u;
            }
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                const uint32_t r = r0 + k * 256u;
                oo[k] = (r < g.B && o[k] <= r) ? ref[o[k]] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k)
                if (r0 + k * 256u < g.B && oo[k] != o[k]) s_ok = 0;  // (a reference forward left oo at "no row")
        }
    }
    __syncthreads();
    if (tid == 0) {
        DecTable D;
        D.valid = s_ok; D.n_used = H.n_used; D.sym_lo = H.sym_lo; D.n_outliers = H.n_esc; D.ebx2 = H.ebx2; D.pad = 0;
        D.ref_off = H.ref_off;
        dtab[t] = D;
        if (!s_ok) set_status(ctrl, DLC_ECORRUPT);
    }
}

// ------------------------------------------------------------------------------------------------
// chunk-parallel decode.  A work-group belongs to one table: it checks the container's header and the table's
// directory entry, rebuilds the canonical code from the stored lengths into an LDS decode table, and then decodes
// `iters` consecutive blocks of NW groups (NW = wavefronts of the work-group), one wavefront per group, lane l walking chunk l.  Each lane keeps
// a 64-bit window of its own bit stream, looks LMAX bits up in the decode table, and the four symbols of a turn
// leave as one 16-byte store (1 KiB contiguous per wavefront instruction).  Nothing is read from a table that fails
// validation.
//
// A lane's symbols hang on one another (the next look-up needs the length of the code before it), so the time a
// group takes is the length of that chain.  The decode table therefore answers for two codewords at a time:
//   entry[i] = single << 31 | adv << 27 | (len1 - 1) << 24 | bin2 << 12 | bin1     for the LMAX-bit string i,
// bin = symbol - R as a signed 12-bit number (what the reconstruction multiplies by 2 * bound); bin1: the codeword
// that prefixes i, len1 its length; bin2: the codeword after it when both fit into the LMAX bits (and len1 <= 8:
// three bits hold it), adv = len1 + len2 then.  Otherwise single = 1 and adv = len1: a second look-up follows,
// rare for the short codes of frequent symbols.
//
// The bit stream words reach the lanes through LDS: every lane copies the next kWin words of its chunk
// into column `lane` of a [kWin][64] staging array of its wavefront (bank = lane, so the lanes never
// collide whatever word each of them is at) and refills its window from there.  The decode loop then
// holds no global load, so nothing in it ever waits for memory: the stores just stream out.
//
// Per table the work-groups add up the escapes they have applied; the last one to finish compares the sum with the
// directory entry (counters in the workspace, zero between calls).
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kWin = 30;                         // staged words per lane (two work-groups share a CU's LDS)
constexpr uint32_t kDecWaves = 8;                     // wavefronts per work-group; 4 or 2 for tables of fewer groups (a
                                                      // destination's piece of a table can be two groups: no idle wavefronts)
constexpr uint32_t kSkipWords = 256 * kW / kV / 32;   // row matching: a bit per row of a group, rows of at least four elements

struct DecScratch {  // lives in the staging area until the decode table is complete
    uint32_t ok;
    uint32_t cl[kLmaxLimit + 2], first[kLmaxLimit + 2], index[kLmaxLimit + 2];
    uint16_t sorted[4096];
    uint16_t one[1 << kLmaxLimit];  // len << 12 | symbol of the codeword that prefixes the LMAX-bit string i
    uint8_t len[4096];
};
// bytes behind the decode table: the staging arrays of the NW wavefronts, or the scratch where that is larger
__host__ __device__ constexpr uint32_t dec_area_bytes(uint32_t nw) {
    return nw * kWin * kW * 4u > (uint32_t)((sizeof(DecScratch) + 15u) & ~15u) ? nw * kWin * kW * 4u : (uint32_t)((sizeof(DecScratch) + 15u) & ~15u);
}

// (len << 12 | symbol) of the codeword that prefixes the LMAX-bit string i: its length is one more than the number of
// limits at or below i (limit[l] = first string that no codeword of length <= l prefixes)
__device__ __forceinline__ uint32_t dec_first_code(const DecScratch& sc, const uint32_t (&limit)[kLmaxLimit + 1], uint32_t i,
                                                   uint32_t LMAX) {
    uint32_t l = 1;
#pragma unroll
    for (uint32_t k = 1; k < (uint32_t)kLmaxLimit; ++k) l += (i >= limit[k]) ? 1u : 0u;
    const uint32_t c = i >> (LMAX - l);
    return (l << 12) | sc.sorted[sc.index[l] + (c - sc.first[l])];
}

template <bool F16, bool VEC, uint32_t NW>
__global__ __launch_bounds__(64 * NW) void k_decode(Geom g, FixedLayout F, const uint8_t* comp, uint64_t comp_bytes,
                                                        Ctrl* ctrl, void* outp, uint32_t wpt, uint32_t iters,
                                                        uint32_t* esc_seen, uint32_t* arrived) {
    constexpr uint32_t kDecThreads = 64u * NW;
    extern __shared__ __align__(16) uint32_t s_lut[];  // [1 << LMAX] decode table, then NW staging arrays
    __shared__ uint32_t s_bad;
    __shared__ unsigned long long s_sum[NW];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t t = blockIdx.x / wpt, b = blockIdx.x % wpt;
    const uint32_t dst = t / g.TD, tl = t - dst * g.TD;  // the container this table is in, and its place there
    comp += (uint64_t)dst * comp_bytes;
    const uint32_t lut_n = 1u << g.LMAX;
    DecScratch& sc = *reinterpret_cast<DecScratch*>(s_lut + lut_n);
    const uint32_t* const goffs = reinterpret_cast<const uint32_t*>(comp + F.off_group);
    const uint32_t n_groups = g.TD * g.G;
    // What a group's decoding starts from sits in the sections whose place the geometry fixes (the host has made
    // sure they lie inside comp_bytes): the loads of the first group go out before anything else is known.
    struct GroupHead { uint32_t cw, goff, gnext; };
    auto group_head = [&](uint32_t grp) {
        GroupHead h;
        const uint32_t gid = tl * g.G + grp;  // group number inside the container
        h.cw = comp[F.off_chunk + (uint64_t)gid * kW + lane];
        h.goff = goffs[gid];
        h.gnext = gid + 1 < n_groups ? goffs[gid + 1] : 0xFFFFFFFFu;  // (the last group ends where the payload does)
        return h;
    };
    const uint32_t grp_first = b * iters * NW + wave;
    GroupHead gh;
    gh.cw = 0; gh.goff = 0; gh.gnext = 0;
    if (grp_first < g.G) gh = group_head(grp_first);
    const DecHead H = dec_validate(g, F, comp, comp_bytes, tl);
    if (tid == 0) { sc.ok = H.ok ? 1u : 0u; s_bad = 0u; }
    if (tid < kLmaxLimit + 2) sc.cl[tid] = 0;
    __syncthreads();
    const uint32_t nl = H.ok ? H.sym_hi - H.sym_lo + 1u : 0u;
    for (uint32_t i = tid; i < nl; i += kDecThreads) {
        const uint32_t l = comp[H.cb + i];
        sc.len[i] = (uint8_t)l;
        if (l > g.LMAX) sc.ok = 0;
        else if (l) atomicAdd(&sc.cl[l], 1u);
    }
    // One group of a wavefront: its words (the chunks', then two per escape) checked against the container, then the
    // lanes' next kWin chunk words fetched into registers.  Branch-free, all loads in flight together: an index past
    // the chunk's end reads its last word instead (an empty chunk reads the word at its position, which still lies
    // inside the container: code-length blocks follow the payload) and is masked to zero when it goes to LDS.
    struct GroupPlace { bool ok; uint32_t n_esc, total; const uint32_t* chunk; };
    auto group_place = [&](const GroupHead& h) {
        GroupPlace P;
        const uint32_t incl = wave_incl_scan(h.cw, lane);
        P.total = __shfl(incl, 63, 64);
        const uint64_t gend = h.gnext == 0xFFFFFFFFu ? H.words_total : (uint64_t)h.gnext;
        P.ok = !(gend > H.words_total || (uint64_t)h.goff + P.total > gend || ((gend - h.goff - P.total) & 1ull));
        P.n_esc = P.ok ? (uint32_t)((gend - h.goff - P.total) >> 1) : 0u;
        P.chunk = reinterpret_cast<const uint32_t*>(comp + F.off_payload) + h.goff + (incl - h.cw);
        return P;
    };
    auto fetch_words = [&](const uint32_t* chunk, uint32_t cw, uint32_t from, uint32_t (&w)[kWin]) {
        const uint32_t last = cw ? cw - 1u : 0u;
#pragma unroll
        for (uint32_t k = 0; k < kWin; ++k) w[k] = chunk[min(from + k, last)];
    };
    uint32_t* const stage = reinterpret_cast<uint32_t*>(s_lut + lut_n) + wave * (kWin * kW) + lane;  // my column
    auto put_words = [&](uint32_t cw, uint32_t from, const uint32_t (&w)[kWin]) {
#pragma unroll
        for (uint32_t k = 0; k < kWin; ++k) stage[k * kW] = from + k < cw ? w[k] : 0u;
    };
    // the first group's words are on their way while the decode table is made
    GroupPlace gp;
    gp.ok = false; gp.n_esc = 0; gp.total = 0; gp.chunk = nullptr;
    uint32_t w_first[kWin];
#pragma unroll
    for (uint32_t k = 0; k < kWin; ++k) w_first[k] = 0;
    if (H.ok && grp_first < g.G) {
        gp = group_place(gh);
        if (gp.ok) fetch_words(gp.chunk, gh.cw, 0, w_first);
    }
    // the container as a whole: its escapes are those of its tables (first work-group of the container)
    if (H.ok && tl == 0 && b == 0) {
        uint32_t part = 0;
        bool big = false;
        for (uint32_t k = tid; k < g.TD; k += kDecThreads) {
            const uint32_t e = reinterpret_cast<const uint32_t*>(comp + kHeaderBytes + (uint64_t)kDirBytes * k)[4];
            big = big || e > g.n;
            part += e > g.n ? 0u : e;
        }
        // (32-bit partial sums per thread cannot wrap: a thread adds at most TD / 512 counts of less than 2^31 each,
        // and TD * n < 2^32 positions in all; across threads they are added as 64-bit values)
        unsigned long long sum = part;
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        if (lane == 0) s_sum[wave] = sum;
        __syncthreads();
        if (tid == 0) {
            unsigned long long all = 0;
            for (uint32_t k = 0; k < NW; ++k) all += s_sum[k];
            if (all != H.n_esc_total) s_bad = 1u;
        }
        if (big) s_bad = 1u;
    }
    __syncthreads();
    const bool ok2 = sc.ok != 0;  // every thread reads the same value, then nobody writes before the barrier
    __syncthreads();
    if (ok2 && H.n_used == 1) {
        if (tid == 0 && (H.sym_lo != H.sym_hi || sc.len[0] != 0)) sc.ok = 0;
        // length 0: every look-up gives one symbol and moves on by nothing
        for (uint32_t i = tid; i < lut_n; i += kDecThreads) s_lut[i] = 0x80000000u | ((H.sym_lo - g.R) & 0xFFFu);
    } else if (ok2) {
        if (wave == 0) {
            // first wavefront: every lane derives the same per-length tables, then the symbols are put in
            // (length, symbol) order, 64 at a time: a symbol's place is the number of symbols of its length before it
            uint64_t kraft = 0;
            uint32_t cnt = 0, code = 0, index = 0;
            uint32_t fill[kLmaxLimit + 1];
#pragma unroll
            for (uint32_t l = 1; l <= (uint32_t)kLmaxLimit; ++l) {
                const uint32_t c = l <= g.LMAX ? sc.cl[l] : 0u;
                kraft += l <= g.LMAX ? (uint64_t)c << (g.LMAX - l) : 0ull;
                cnt += c;
                code <<= 1;
                if (lane == 0) { sc.first[l] = code; sc.index[l] = index; }
                fill[l] = index;
                code += c;
                index += c;
            }
            if (kraft != (1ull << g.LMAX) || cnt != H.n_used) {
                if (lane == 0) sc.ok = 0;
            } else {
                const uint64_t below = (1ull << lane) - 1ull;
                for (uint32_t base = 0; base < nl; base += 64) {
                    const uint32_t i = base + lane;
                    const uint32_t L = i < nl ? sc.len[i] : 0u;
                    if (__ballot(L != 0u) == 0ull) continue;  // (a stretch of unused symbols: the escape symbol's code can lie far below the others)
#pragma unroll
                    for (uint32_t l = 1; l <= (uint32_t)kLmaxLimit; ++l) {
                        const uint64_t m = __ballot(L == l);
                        if (L == l) sc.sorted[fill[l] + (uint32_t)__popcll(m & below)] = (uint16_t)(H.sym_lo + i);
                        fill[l] += (uint32_t)__popcll(m);
                    }
                }
            }
        }
        __syncthreads();
        if (sc.ok != 0) {
            // the LMAX-bit string i starts with a codeword of length l iff i < limit[l] and not already
            // i < limit[l-1]; the limits are the same for every thread (scalar registers).  A thread fills eight
            // strings in a row: all of them start with one codeword when they agree down to its last bit, which for
            // the short codes that cover most of the table is the rule.
            uint32_t limit[kLmaxLimit + 1];
#pragma unroll
            for (uint32_t l = 1; l <= (uint32_t)kLmaxLimit; ++l)
                limit[l] = l <= g.LMAX ? (sc.first[l] + sc.cl[l]) << (g.LMAX - l) : 0xFFFFFFFFu;
            for (uint32_t i0 = tid * 8u; i0 < lut_n; i0 += kDecThreads * 8u) {  // (lut_n >= 16: a multiple of 8)
                const uint32_t ea = dec_first_code(sc, limit, i0, g.LMAX), la = ea >> 12;
                uint32_t e[8];
                if (g.LMAX - la >= 3u) {
#pragma unroll
                    for (uint32_t k = 0; k < 8; ++k) e[k] = ea;
                } else {
                    e[0] = ea;
#pragma unroll
                    for (uint32_t k = 1; k < 8; ++k) e[k] = dec_first_code(sc, limit, i0 + k, g.LMAX);
                }
                uint4 v;
                v.x = e[0] | (e[1] << 16); v.y = e[2] | (e[3] << 16); v.z = e[4] | (e[5] << 16); v.w = e[6] | (e[7] << 16);
                *reinterpret_cast<uint4*>(&sc.one[i0]) = v;
            }
            __syncthreads();  // (uniform: sc.ok was read after a barrier and nothing has written it since)
            for (uint32_t i = tid; i < lut_n; i += kDecThreads) {
                const uint32_t e1 = sc.one[i], l1 = e1 >> 12;
                const uint32_t e2 = sc.one[(i << l1) & (lut_n - 1u)], l2 = e2 >> 12;  // what follows the first codeword
                const bool both = l1 + l2 <= g.LMAX && l1 <= 8u;  // the second codeword lies inside the LMAX bits too
                const uint32_t q1 = ((e1 & 0xFFFu) - g.R) & 0xFFFu, q2 = ((e2 & 0xFFFu) - g.R) & 0xFFFu;
                s_lut[i] = both ? ((l1 + l2) << 27) | ((l1 - 1u) << 24) | (q2 << 12) | q1 : 0x80000000u | (l1 << 27) | q1;
            }
        }
    }
    __syncthreads();
    const bool valid = sc.ok != 0;
    __syncthreads();  // the scratch is staging memory from here on
    uint32_t my_esc = 0;   // escapes this wavefront has applied (uniform)
    bool bad = false;      // something in this wavefront's groups does not add up
    if (valid) {
        const float ebx2 = H.ebx2;
        const uint32_t lshift = 32u - g.LMAX;
        uint8_t* tab = static_cast<uint8_t*>(outp) + (size_t)t * g.n * g.es;
        const uint32_t turns = g.S / kV;
        const uint32_t* const ref = H.ref_off ? reinterpret_cast<const uint32_t*>(comp + H.ref_off) : nullptr;
        uint32_t* const skipbits = reinterpret_cast<uint32_t*>(s_lut + lut_n) + dec_area_bytes(NW) / 4u + wave * kSkipWords;
        for (uint32_t it = 0; it < iters; ++it) {
            const uint32_t grp = grp_first + it * NW;
            if (grp >= g.G) break;  // whole wavefront
            // A lane's place in its bit stream: the two words w0, w1 it is decoding from, `c` bits of w0 already used
            // (0..31), the word after them in `nxt`, fetched ahead from the staging rows; kr = staging row of `nxt`,
            // wbase = chunk word index of staging row 0.
            uint32_t wbase = 0, kr = 0;
            if (it == 0) {
                if (gp.ok) put_words(gh.cw, 0, w_first);
            } else {
                gh = group_head(grp);
                gp = group_place(gh);
                if (gp.ok) {
                    uint32_t w[kWin];
                    fetch_words(gp.chunk, gh.cw, 0, w);
                    put_words(gh.cw, 0, w);
                }
            }
            if (!gp.ok) {
                bad = true;
                continue;
            }
            const uint32_t cw = gh.cw, n_esc = gp.n_esc, total = gp.total;
            const uint32_t* const chunk = gp.chunk;
            // the words from `nxt` on, anew, so that `nxt` is row 0
            // more = words of the chunk past row 0 of the staging rows, less one: a lane needs new rows when `nxt` is
            // among the last two rows (a turn moves at most two words on) and kr < more
            int more = (int)cw - 1;
            auto restage = [&]() {
                wbase += kr;
                more -= (int)kr;
                kr = 0;
                uint32_t w[kWin];
                fetch_words(chunk, cw, wbase, w);
                put_words(cw, wbase, w);
            };
            uint32_t w0 = stage[0], w1 = stage[kW], nxt = stage[2u * kW], c = 0;
            kr = 2;
            const uint32_t base = grp * (kW * g.S) + lane * kV;
            // row matching: which rows of this group refer to another row, as a bit per row in LDS (at most 64*S/4 rows)
            const uint32_t row_lo = (grp * (kW * g.S)) / g.D;
            if (ref != nullptr) {
                const uint32_t last_el = min(g.n, (grp + 1u) * (kW * g.S)) - 1u;
                const uint32_t n_rows = last_el / g.D - row_lo + 1u;  // <= 64*S/4 because dim % 4 == 0 here
                for (uint32_t r0 = 0; r0 < n_rows; r0 += 64) {  // uniform trip count
                    const uint32_t r = r0 + lane;
                    const bool refers = r < n_rows && ref[row_lo + r] != row_lo + r;
                    const uint64_t m = __ballot(refers);
                    if (lane == 0) { skipbits[r0 / 32u] = (uint32_t)m; skipbits[r0 / 32u + 1u] = (uint32_t)(m >> 32); }
                }
                __builtin_amdgcn_wave_barrier();
            }
            for (uint32_t j = 0; j < turns; ++j) {
                const uint32_t idx = base + j * (kW * kV);
                // a turn moves at most two more words; restage (whole wavefront) when a lane that still has words to
                // fetch could run off its rows
                if (__ballot(kr >= kWin - 2u && (int)kr < more) != 0ull) restage();
                bool coded = idx < g.n;
                if (ref != nullptr && coded) {  // a row that refers to another has no bits in the stream; it is copied afterwards
                    const uint32_t r = idx / g.D - row_lo;
                    coded = ((skipbits[r >> 5] >> (r & 31u)) & 1u) == 0u;
                }
                if (coded) {
                    float v4[4];
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) {
                        const uint64_t win = (((uint64_t)w0 << 32) | w1) << c;  // the stream from the lane's place on
                        const uint32_t e = s_lut[(uint32_t)(win >> 32) >> lshift];
                        uint32_t adv = (e >> 27) & 15u;
                        int q2 = (int)(e << 8) >> 20;
                        if (__ballot((int)e < 0) != 0ull) {  // an entry that answers for one codeword only: the next one by a look-up of its own
                            const uint32_t e2 = s_lut[(uint32_t)((win << adv) >> 32) >> lshift];
                            if ((int)e < 0) {
                                q2 = (int)(e2 << 20) >> 20;
                                adv += (int)e2 < 0 ? (e2 >> 27) & 15u : ((e2 >> 24) & 7u) + 1u;
                            }
                        }
                        if constexpr (!VEC) {  // a turn can reach past the table's end: such a position has no bits
                            if (idx + (uint32_t)(h2 * 2) + 1u >= g.n) {
                                const uint32_t l1 = (int)e < 0 ? (e >> 27) & 15u : ((e >> 24) & 7u) + 1u;
                                adv = idx + (uint32_t)(h2 * 2) < g.n ? l1 : 0u;
                            }
                        }
                        c += adv;
                        // past the end of w0: move on by a word (the row after `nxt` is read whether or not: same value then)
                        const bool step = c > 31u;
                        w0 = step ? w1 : w0;
                        w1 = step ? nxt : w1;
                        c &= 31u;
                        kr += step ? 1u : 0u;
                        nxt = stage[min(kr, kWin - 1u) * kW];  // (rows past the chunk's end are zero)
                        v4[h2 * 2] = (float)((int)(e << 20) >> 20) * ebx2;
                        v4[h2 * 2 + 1] = (float)q2 * ebx2;
                    }
                    // streaming stores: the output is written once and is larger than the caches
                    if constexpr (VEC) {
                        if constexpr (F16) {
                            typedef uint32_t u2v __attribute__((ext_vector_type(2)));
                            u2v o;
                            o.x = (uint32_t)__half_as_ushort(half_rne(v4[0])) |
                                  ((uint32_t)__half_as_ushort(half_rne(v4[1])) << 16);
                            o.y = (uint32_t)__half_as_ushort(half_rne(v4[2])) |
                                  ((uint32_t)__half_as_ushort(half_rne(v4[3])) << 16);
                            __builtin_nontemporal_store(o, reinterpret_cast<u2v*>(reinterpret_cast<uint16_t*>(tab) + idx));
                        } else {
                            typedef float f4v __attribute__((ext_vector_type(4)));
                            f4v o4 = {v4[0], v4[1], v4[2], v4[3]};
                            __builtin_nontemporal_store(o4, reinterpret_cast<f4v*>(reinterpret_cast<float*>(tab) + idx));
                        }
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (idx + v < g.n) {
                                if constexpr (F16) reinterpret_cast<__half*>(tab)[idx + v] = half_rne(v4[v]);
                                else reinterpret_cast<float*>(tab)[idx + v] = v4[v];
                            }
                    }
                }
            }
            // a chunk's codewords end inside its words: w0 is chunk word wbase + kr - 2, and c of its bits are used
            if (__ballot(32u * (wbase + kr - 2u) + c > 32u * cw) != 0ull) bad = true;
            if (n_esc != 0u) {  // uniform over the wavefront: verbatim values over the decoded placeholders
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_s_waitcnt(0);  // the wavefront's own stores above are out before the overwrites below
                const uint32_t* rec = reinterpret_cast<const uint32_t*>(comp + F.off_payload) + gh.goff + total;
                const uint32_t lo = grp * (kW * g.S);
                const uint32_t hi = min(g.n, lo + kW * g.S);
                bool off_range = false;
                for (uint32_t r = lane; r < n_esc; r += 64) {
                    const uint32_t idx = rec[2u * r], raw = rec[2u * r + 1];
                    if (idx < lo || idx >= hi) { off_range = true; continue; }
                    if constexpr (F16) reinterpret_cast<uint16_t*>(tab)[idx] = (uint16_t)raw;
                    else reinterpret_cast<uint32_t*>(tab)[idx] = raw;
                }
                if (__ballot(off_range) != 0ull) bad = true;
                my_esc += n_esc;
            }
        }
        if (my_esc != 0u && lane == 0) {
            __hip_atomic_fetch_add(&esc_seen[t], my_esc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // counted before the work-group says it is done
        }
    }
    if (bad && lane == 0) s_bad = 1u;
    __syncthreads();
    if (tid == 0) {
        bool corrupt = !valid || s_bad != 0u;
        // the last work-group of the table: all escapes of the table have been seen
        if (__hip_atomic_fetch_add(&arrived[t], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == wpt) {
            const uint32_t seen = __hip_atomic_exchange(&esc_seen[t], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&arrived[t], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (valid && seen != H.n_esc) corrupt = true;
        }
        if (corrupt) set_status(ctrl, DLC_ECORRUPT);
    }
}

// rows that refer to an earlier row of their table: copies of that row's reconstruction (after the decode kernel).
// A thread per 16-byte (fp32) / 8-byte (fp16) piece of a row, pieces of a row on neighbouring threads.
template <typename U>
__global__ __launch_bounds__(256) void k_row_copy(Geom g, const uint8_t* comp, uint64_t comp_bytes, const DecTable* dtab,
                                                  void* outp) {
    const uint32_t t = blockIdx.y;
    const uint32_t dst = t / g.TD;  // the container this table is in
    comp += (uint64_t)dst * comp_bytes;
    const DecTable D = dtab[t];
    if (!D.valid || D.ref_off == 0) return;  // uniform
    const uint32_t* ref = reinterpret_cast<const uint32_t*>(comp + D.ref_off);
    U* tab = reinterpret_cast<U*>(static_cast<uint8_t*>(outp) + (size_t)t * g.n * g.es);
    const uint32_t upr = g.D / 4u;  // pieces per row (four elements each; dim % 4 == 0)
    const uint32_t total = g.B * upr;
    // four pieces a thread has in flight: references first, then the rows they point at (named variables, not an
    // array: the compiler moved an array of vectors into LDS)
    const uint32_t stride = gridDim.x * 256;
    for (uint32_t i0 = blockIdx.x * 256 + threadIdx.x; i0 < total; i0 += stride * 4u) {
        uint32_t row[4], o[4];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            const uint32_t i = i0 + k * stride;
            row[k] = i < total ? i / upr : 0xFFFFFFFFu;
            o[k] = i < total ? ref[row[k]] : 0xFFFFFFFFu;
        }
        auto src = [&](uint32_t k) -> size_t { return (size_t)o[k] * upr + (i0 + k * stride - row[k] * upr); };
        U v0{}, v1{}, v2{}, v3{};
        if (o[0] != row[0]) v0 = tab[src(0)];
        if (o[1] != row[1]) v1 = tab[src(1)];
        if (o[2] != row[2]) v2 = tab[src(2)];
        if (o[3] != row[3]) v3 = tab[src(3)];
        if (o[0] != row[0]) tab[(size_t)i0] = v0;
        if (o[1] != row[1]) tab[(size_t)i0 + stride] = v1;
        if (o[2] != row[2]) tab[(size_t)i0 + 2u * stride] = v2;
        if (o[3] != row[3]) tab[(size_t)i0 + 3u * stride] = v3;
    }
}

hipError_t launch_decompress(const Geom& g, const uint8_t* comp, uint64_t comp_bytes, void* out, const Ws& w, int pl,
                             void* prof, hipStream_t s) {
    const bool f16 = g.dtype == DLC_F16;
    const FixedLayout F = fixed_layout(g);
    if (g.lz)  // before the decode kernel: the row-copy kernel follows the references only where they were checked
        hipLaunchKernelGGL(k_dec_refs, dim3(g.T), dim3(256), 0, s, g, F, comp, comp_bytes, w.dtab, w.ctrl);
    {
        // a work-group decodes `iters` blocks of nw groups of one table, a wavefront each: enough blocks to spread the
        // cost of its decode table, enough work-groups (a few thousand) to fill the chip whatever the shape, and no
        // more wavefronts than a table has groups
        const uint32_t nw = g.G >= 6u ? kDecWaves : (g.G >= 3u ? 4u : 2u);
        const uint32_t bpt = (g.G + nw - 1) / nw;
        const uint64_t blocks = (uint64_t)g.T * bpt;
        const uint32_t iters = (uint32_t)std::min<uint64_t>(4, std::max<uint64_t>(1, blocks / 2048));
        const uint32_t wpt = (bpt + iters - 1) / iters;  // work-groups per table
        dim3 grid(g.T * wpt), block(64 * nw);
        const size_t sm = ((size_t)4 << g.LMAX) + dec_area_bytes(nw) + (g.lz ? (size_t)nw * kSkipWords * 4 : 0);
        if (prof_on(pl, P_DECODE)) prof_begin(prof, P_DECODE, s);
#define DLC_DEC2(FF, V, N) hipLaunchKernelGGL((k_decode<FF, V, N>), grid, block, sm, s, g, F, comp, (uint64_t)comp_bytes, w.ctrl, out, wpt, iters, w.dec_esc, w.dec_arrive)
#define DLC_DEC(FF, V) do { if (nw == 8u) DLC_DEC2(FF, V, 8u); else if (nw == 4u) DLC_DEC2(FF, V, 4u); else DLC_DEC2(FF, V, 2u); } while (0)
        if (f16) { if (g.vec) DLC_DEC(true, true); else DLC_DEC(true, false); }
        else { if (g.vec) DLC_DEC(false, true); else DLC_DEC(false, false); }
#undef DLC_DEC
#undef DLC_DEC2
        if (g.lz) {
            const uint32_t bx = std::min<uint32_t>((g.B * (g.D / 4u) + 255u) / 256u, 256u);
            if (f16) hipLaunchKernelGGL(k_row_copy<uint2>, dim3(bx, g.T), dim3(256), 0, s, g, comp, (uint64_t)comp_bytes, w.dtab, out);
            else hipLaunchKernelGGL(k_row_copy<uint4>, dim3(bx, g.T), dim3(256), 0, s, g, comp, (uint64_t)comp_bytes, w.dtab, out);
        }
        if (prof_on(pl, P_DECODE)) prof_end(prof, P_DECODE, s);
    }
    return hipGetLastError();
}

template <uint32_t NW>
static hipError_t decode_set_attributes() {
    const int bytes = (4 << kLmaxLimit) + (int)dec_area_bytes(NW) + (int)(NW * kSkipWords * 4);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_decode<false, false, NW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_decode<false, true, NW>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_decode<true, false, NW>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_decode<true, true, NW>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    return e;
}

hipError_t decompress_set_attributes() {
    hipError_t e = decode_set_attributes<8u>();
    if (e == hipSuccess) e = decode_set_attributes<4u>();
    if (e == hipSuccess) e = decode_set_attributes<2u>();
    return e;
}

}  // namespace dlc
