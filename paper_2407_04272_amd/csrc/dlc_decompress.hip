// Decompression kernels for gfx950: container validation + decode tables, chunk-parallel decode,
// escape scatter.
#include <algorithm>

#include "dlc_internal.h"

namespace dlc {

__device__ __forceinline__ uint64_t d_a16(uint64_t x) { return (x + 15ull) & ~15ull; }

// ------------------------------------------------------------------------------------------------
// One work-group per table (of every container, when there are several): checks the header against the context's geometry and the table's
// directory entry against the header, rebuilds the canonical code from the stored lengths and fills
// the table's decode table: entry[i] = len << 12 | symbol for the codeword that prefixes the LMAX-bit
// string i.  Anything inconsistent marks the table (or the whole container) invalid.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_dec_prepare(Geom g, const uint8_t* comp, uint64_t comp_bytes, uint16_t* lut,
                                                     DecLayout* dlay, DecTable* dtab, Ctrl* ctrl) {
    __shared__ uint32_t s_ok;
    __shared__ uint32_t s_cl[kLmaxLimit + 2], s_first[kLmaxLimit + 2], s_index[kLmaxLimit + 2];
    __shared__ uint16_t s_sorted[4096];
    __shared__ uint8_t s_len[4096];
    const uint32_t tid = threadIdx.x, t = blockIdx.x;
    // the container this table is in: container d starts at d * comp_bytes (comp_bytes: the room of one container)
    const uint32_t dst = t / g.TD, tl = t - dst * g.TD;
    comp += (uint64_t)dst * comp_bytes;
    const uint32_t* h = reinterpret_cast<const uint32_t*>(comp);
    const uint64_t* q = reinterpret_cast<const uint64_t*>(comp);
    DecLayout L;
    bool ok = comp_bytes >= kHeaderBytes + (uint64_t)kDirBytes * g.TD;
    if (ok) {
        ok = h[H_MAGIC] == kMagic && h[H_VERSION] == kVersion && h[H_DTYPE] == g.dtype && h[H_T] == g.TD &&
             h[H_B] == g.B && h[H_D] == g.D && h[H_R] == g.R && h[H_S] == g.S && h[H_LMAX] == g.LMAX &&
             h[H_W] == kW && h[H_V] == kV && h[H_NG] == g.TD * g.G;
    }
    uint64_t off_cb = 0, n_out = 0, total = 0;
    if (ok) {
        const FixedLayout F = fixed_layout(g);
        n_out = q[HQ_NOUT];
        L.words_total = q[HQ_WORDS];
        L.off_group = q[HQ_OFF_GROUP]; L.off_chunk = q[HQ_OFF_CHUNK]; L.off_payload = q[HQ_OFF_PAYLOAD];
        off_cb = q[HQ_OFF_CB];
        total = q[HQ_TOTAL];
        ok = total <= comp_bytes && L.off_group == F.off_group && L.off_chunk == F.off_chunk &&
             L.off_payload == F.off_payload && L.words_total <= 0xFFFFFFFFull && n_out <= (uint64_t)g.n * g.TD &&
             off_cb == d_a16(L.off_payload + 4ull * L.words_total) && total >= off_cb;
    }
    if (tl == 0 && tid == 0) {
        L.valid = ok; L.pad = 0;
        dlay[dst] = L;
        if (!ok) set_status(ctrl, DLC_ECORRUPT);
    }
    DecTable D;
    D.valid = 0; D.n_used = 0; D.sym_lo = 0; D.n_outliers = 0; D.ebx2 = 0.f; D.pad = 0; D.ref_off = 0;
    uint32_t sym_lo = 0, sym_hi = 0, n_used = 0;
    uint64_t cb = 0;
    if (ok) {
        const uint8_t* d = comp + kHeaderBytes + (uint64_t)kDirBytes * tl;
        const uint32_t* d32 = reinterpret_cast<const uint32_t*>(d);
        const uint64_t* d64 = reinterpret_cast<const uint64_t*>(d + 24);
        const float eb = __uint_as_float(d32[0]);
        n_used = d32[1]; sym_lo = d32[2]; sym_hi = d32[3];
        D.n_outliers = d32[4];
        cb = d64[0];
        ok = eb > 0.f && eb < __builtin_inff() && d32[5] == g.G && sym_lo <= sym_hi && sym_hi < g.K && n_used >= 1 &&
             n_used <= sym_hi - sym_lo + 1u && cb >= off_cb && cb + (sym_hi - sym_lo + 1u) <= total &&
             D.n_outliers <= g.n;
        D.ebx2 = eb * 2.0f;
        D.sym_lo = sym_lo;
        D.n_used = n_used;
        // row matching: references behind the code-length blocks (only a context made for it decodes them, and the
        // kernels want a lane's four elements in one row)
        D.ref_off = d64[1];
        if (D.ref_off != 0)
            ok = ok && g.lz != 0 && (g.D % 4u) == 0 && (D.ref_off % 4u) == 0 && D.ref_off >= off_cb &&
                 D.ref_off + 4ull * g.B <= total;
    }
    if (tid == 0) s_ok = ok;
    if (tid < kLmaxLimit + 2) s_cl[tid] = 0;
    __syncthreads();
    if (ok && D.ref_off != 0) {  // every reference points back, at a row that is coded
        const uint32_t* ref = reinterpret_cast<const uint32_t*>(comp + D.ref_off);
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
    const uint32_t nl = ok ? sym_hi - sym_lo + 1u : 0u;
    for (uint32_t i = tid; i < nl; i += 256) {
        const uint32_t l = comp[cb + i];
        s_len[i] = (uint8_t)l;
        if (l > g.LMAX) s_ok = 0;
        else if (l) atomicAdd(&s_cl[l], 1u);
    }
    __syncthreads();
    const bool ok2 = s_ok != 0;  // every thread reads the same value, then nobody writes before the barrier
    __syncthreads();
    uint16_t* my_lut = lut + ((size_t)t << g.LMAX);
    const uint32_t lut_n = 1u << g.LMAX;
    if (ok2 && n_used == 1) {
        if (tid == 0 && (sym_lo != sym_hi || s_len[0] != 0)) s_ok = 0;
        for (uint32_t i = tid; i < lut_n; i += 256) my_lut[i] = (uint16_t)sym_lo;  // length 0
    } else if (ok2) {
        if (tid < 64) {
            // first wavefront: every lane derives the same per-length tables, then the symbols are put in
            // (length, symbol) order, 64 at a time: a symbol's place is the number of symbols of its length before it
            const uint32_t lane = tid;
            uint64_t kraft = 0;
            uint32_t cnt = 0, code = 0, index = 0;
            uint32_t fill[kLmaxLimit + 1];
#pragma unroll
            for (uint32_t l = 1; l <= (uint32_t)kLmaxLimit; ++l) {
                const uint32_t c = l <= g.LMAX ? s_cl[l] : 0u;
                kraft += l <= g.LMAX ? (uint64_t)c << (g.LMAX - l) : 0ull;
                cnt += c;
                code <<= 1;
                if (lane == 0) { s_first[l] = code; s_index[l] = index; }
                fill[l] = index;
                code += c;
                index += c;
            }
            if (kraft != (1ull << g.LMAX) || cnt != n_used) {
                if (lane == 0) s_ok = 0;
            } else {
                const uint64_t below = (1ull << lane) - 1ull;
                for (uint32_t base = 0; base < nl; base += 64) {
                    const uint32_t i = base + lane;
                    const uint32_t L = i < nl ? s_len[i] : 0u;
#pragma unroll
                    for (uint32_t l = 1; l <= (uint32_t)kLmaxLimit; ++l) {
                        const uint64_t m = __ballot(L == l);
                        if (L == l) s_sorted[fill[l] + (uint32_t)__popcll(m & below)] = (uint16_t)(sym_lo + i);
                        fill[l] += (uint32_t)__popcll(m);
                    }
                }
            }
        }
        __syncthreads();
        const bool ok3 = s_ok != 0;
        if (ok3) {
            // the LMAX-bit string i starts with a codeword of length l iff i < limit[l] and not already
            // i < limit[l-1]; the limits are the same for every thread (scalar registers)
            uint32_t limit[kLmaxLimit + 1];
#pragma unroll
            for (uint32_t l = 1; l <= (uint32_t)kLmaxLimit; ++l)
                limit[l] = l <= g.LMAX ? (s_first[l] + s_cl[l]) << (g.LMAX - l) : 0xFFFFFFFFu;
            for (uint32_t i = tid; i < lut_n; i += 256) {
                uint32_t l = 1;
#pragma unroll
                for (uint32_t k = 1; k < (uint32_t)kLmaxLimit; ++k) l += (i >= limit[k]) ? 1u : 0u;
                const uint32_t c = i >> (g.LMAX - l);
                my_lut[i] = (uint16_t)((l << 12) | s_sorted[s_index[l] + (c - s_first[l])]);
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        D.valid = s_ok;
        dtab[t] = D;
        if (!s_ok) set_status(ctrl, DLC_ECORRUPT);
    }
}

// ------------------------------------------------------------------------------------------------
// chunk-parallel decode: one wavefront per group, lane l walks chunk l.  Each lane keeps a 64-bit
// window of its own bit stream, looks LMAX bits up in the table's LDS decode table, and the four
// symbols of a turn leave as one 16-byte store (1 KiB contiguous per wavefront instruction).
//
// The bit stream words reach the lanes through LDS: every lane copies the next kWin words of its chunk
// into column `lane` of a [kWin][64] staging array of its wavefront (bank = lane, so the lanes never
// collide whatever word each of them is at) and refills its window from there.  The decode loop then
// holds no global load, so nothing in it ever waits for memory: the stores just stream out.
// ------------------------------------------------------------------------------------------------
#ifndef DLC_DEC_WIN
#define DLC_DEC_WIN 32
#endif
#ifndef DLC_DEC_WAVES
#define DLC_DEC_WAVES 8
#endif
constexpr uint32_t kWin = DLC_DEC_WIN;            // staged words per lane
constexpr uint32_t kDecWaves = DLC_DEC_WAVES;        // wavefronts per work-group
constexpr uint32_t kSkipWords = 256 * kW / kV / 32;   // row matching: a bit per row of a group, rows of at least four elements

template <bool F16, bool VEC>
__global__ __launch_bounds__(64 * DLC_DEC_WAVES) void k_decode(Geom g, const uint8_t* comp, const uint16_t* lut, const DecLayout* dlay,
                                                const DecTable* dtab, Ctrl* ctrl, void* outp, uint32_t bpt, uint64_t comp_stride) {
    extern __shared__ __align__(16) uint16_t s_lut[];  // [1 << LMAX] decode table, then kDecWaves staging arrays
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t t = blockIdx.x / bpt, b = blockIdx.x % bpt;
    const uint32_t dst = t / g.TD, tl = t - dst * g.TD;  // the container this table is in, and its place there
    comp += (uint64_t)dst * comp_stride;
    const DecLayout L = dlay[dst];
    const DecTable D = dtab[t];
    if (!L.valid || !D.valid) return;  // uniform over the work-group
    const uint32_t lut_n = 1u << g.LMAX;
    {
        const uint4* src = reinterpret_cast<const uint4*>(lut + ((size_t)t << g.LMAX));
        uint4* dst = reinterpret_cast<uint4*>(s_lut);
        for (uint32_t i = tid; i < lut_n / 8; i += 64 * kDecWaves) dst[i] = src[i];
    }
    __syncthreads();
    const uint32_t grp = b * kDecWaves + wave;
    if (grp >= g.G) return;  // whole wavefront; no barrier follows
    uint32_t* stage = reinterpret_cast<uint32_t*>(s_lut + lut_n) + wave * (kWin * kW) + lane;  // my column
    const uint32_t gid = tl * g.G + grp;  // group number inside the container
    const uint32_t cw = comp[L.off_chunk + (uint64_t)gid * kW + lane];
    const uint32_t incl = wave_incl_scan(cw, lane);
    const uint32_t total = __shfl(incl, 63, 64);
    const uint32_t* goffs = reinterpret_cast<const uint32_t*>(comp + L.off_group);
    const uint64_t goff = goffs[gid];
    const uint64_t gend = gid + 1 < g.TD * g.G ? (uint64_t)goffs[gid + 1] : L.words_total;
    // the group's words: its chunks, then two words per escape
    if (gend > L.words_total || goff + total > gend || ((gend - goff - total) & 1ull)) {
        if (lane == 0) set_status(ctrl, DLC_ECORRUPT);
        return;
    }
    const uint32_t n_esc = (uint32_t)((gend - goff - total) >> 1);
    const uint32_t* chunk = reinterpret_cast<const uint32_t*>(comp + L.off_payload) + goff + (incl - cw);
    uint32_t taken = 0;   // words of the chunk already moved into buf
    uint32_t wbase = 0;   // chunk word index of staging row 0
    // stage words [wbase, wbase + kWin) of my chunk (zero past its end).  Branch-free, all loads in flight
    // together: an index past the end reads the chunk's last word instead (an empty chunk reads the word at
    // its position, which still lies inside the container: code-length blocks follow the payload) and is
    // masked to zero.
    const uint32_t last = cw ? cw - 1u : 0u;
    auto restage = [&]() {
        wbase = taken;
        uint32_t w[kWin];
#pragma unroll
        for (uint32_t k = 0; k < kWin; ++k) w[k] = chunk[min(wbase + k, last)];
#pragma unroll
        for (uint32_t k = 0; k < kWin; ++k) stage[k * kW] = wbase + k < cw ? w[k] : 0u;
    };
    restage();
    uint64_t buf = ((uint64_t)stage[0] << 32) | stage[kW];
    taken = 2;
    uint32_t nb = 64;  // bits of buf in use (bits past the end of the chunk read as zero)
    const float ebx2 = D.ebx2;
    const int R = (int)g.R;
    const uint32_t shift = 64u - g.LMAX;
    uint8_t* tab = static_cast<uint8_t*>(outp) + (size_t)t * g.n * g.es;
    const uint32_t base = grp * (kW * g.S) + lane * kV;
    const uint32_t turns = g.S / kV;
    // row matching: which rows of this group refer to another row, as a bit per row in LDS (at most 64*S/4 rows)
    const uint32_t* const ref = D.ref_off ? reinterpret_cast<const uint32_t*>(comp + D.ref_off) : nullptr;
    uint32_t* const skipbits = reinterpret_cast<uint32_t*>(s_lut + lut_n) + kDecWaves * (kWin * kW) + wave * kSkipWords;
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
        // a turn takes at most two more words; restage (whole wavefront) when a lane could run off its rows
        if (__ballot(taken + 2u > wbase + kWin && taken < cw) != 0ull) restage();
        bool coded = idx < g.n;
        if (ref != nullptr && coded) {  // a row that refers to another has no bits in the stream; it is copied afterwards
            const uint32_t r = idx / g.D - row_lo;
            coded = ((skipbits[r >> 5] >> (r & 31u)) & 1u) == 0u;
        }
        if (coded) {
            float v4[4];
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                if (nb <= 32u) {
                    const uint32_t k = taken - wbase;  // < kWin by the restage rule (rows past the chunk's end are zero)
                    buf |= (uint64_t)stage[(k < kWin ? k : kWin - 1u) * kW] << (32u - nb);
                    nb += 32u;
                    ++taken;
                }
#pragma unroll
                for (int v = 0; v < 2; ++v) {
                    const uint32_t e = s_lut[(uint32_t)(buf >> shift)];
                    const uint32_t len = e >> 12;
                    buf <<= len;
                    nb -= len;
                    v4[h2 * 2 + v] = (float)((int)(e & 0xFFFu) - R) * ebx2;
                }
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
    if (n_esc != 0u) {  // uniform over the wavefront: verbatim values over the decoded placeholders
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_s_waitcnt(0);  // the wavefront's own stores above are out before the overwrites below
        const uint32_t* rec = reinterpret_cast<const uint32_t*>(comp + L.off_payload) + goff + total;
        const uint32_t lo = grp * (kW * g.S);
        const uint32_t hi = min(g.n, lo + kW * g.S);
        for (uint32_t r = lane; r < n_esc; r += 64) {
            const uint32_t idx = rec[2u * r], raw = rec[2u * r + 1];
            if (idx < lo || idx >= hi) { set_status(ctrl, DLC_ECORRUPT); continue; }
            if constexpr (F16) reinterpret_cast<uint16_t*>(tab)[idx] = (uint16_t)raw;
            else reinterpret_cast<uint32_t*>(tab)[idx] = raw;
        }
    }
}

// rows that refer to an earlier row of their table: copies of that row's reconstruction (after the decode kernel).
// A thread per 16-byte (fp32) / 8-byte (fp16) piece of a row, pieces of a row on neighbouring threads.
template <typename U>
__global__ __launch_bounds__(256) void k_row_copy(Geom g, const uint8_t* comp, uint64_t comp_bytes, const DecLayout* dlay,
                                                  const DecTable* dtab, void* outp) {
    const uint32_t t = blockIdx.y;
    const uint32_t dst = t / g.TD;  // the container this table is in
    comp += (uint64_t)dst * comp_bytes;
    const DecTable D = dtab[t];
    if (!dlay[dst].valid || !D.valid || D.ref_off == 0) return;  // uniform
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
    if (prof_on(pl, P_DEC_PREPARE)) prof_begin(prof, P_DEC_PREPARE, s);
    hipLaunchKernelGGL(k_dec_prepare, dim3(g.T), dim3(256), 0, s, g, comp, comp_bytes, w.lut, w.dlay, w.dtab, w.ctrl);
    if (prof_on(pl, P_DEC_PREPARE)) prof_end(prof, P_DEC_PREPARE, s);
    {
        const uint32_t bpt = (g.G + kDecWaves - 1) / kDecWaves;
        dim3 grid(g.T * bpt), block(64 * kDecWaves);
        const size_t sm = ((size_t)2 << g.LMAX) + (size_t)kDecWaves * kWin * kW * 4 + (g.lz ? (size_t)kDecWaves * kSkipWords * 4 : 0);
        if (prof_on(pl, P_DECODE)) prof_begin(prof, P_DECODE, s);
#define DLC_DEC(F, V) hipLaunchKernelGGL((k_decode<F, V>), grid, block, sm, s, g, comp, w.lut, w.dlay, w.dtab, w.ctrl, out, bpt, (uint64_t)comp_bytes)
        if (f16) { if (g.vec) DLC_DEC(true, true); else DLC_DEC(true, false); }
        else { if (g.vec) DLC_DEC(false, true); else DLC_DEC(false, false); }
#undef DLC_DEC
        if (g.lz) {
            const uint32_t bx = std::min<uint32_t>((g.B * (g.D / 4u) + 255u) / 256u, 256u);
            if (f16) hipLaunchKernelGGL(k_row_copy<uint2>, dim3(bx, g.T), dim3(256), 0, s, g, comp, (uint64_t)comp_bytes, w.dlay, w.dtab, out);
            else hipLaunchKernelGGL(k_row_copy<uint4>, dim3(bx, g.T), dim3(256), 0, s, g, comp, (uint64_t)comp_bytes, w.dlay, w.dtab, out);
        }
        if (prof_on(pl, P_DECODE)) prof_end(prof, P_DECODE, s);
    }
    return hipGetLastError();
}

hipError_t decompress_set_attributes() {
    const int bytes = (2 << kLmaxLimit) + (int)(kDecWaves * kWin * kW * 4) + (int)(kDecWaves * kSkipWords * 4);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_decode<false, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_decode<false, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_decode<true, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_decode<true, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    return e;
}

}  // namespace dlc
