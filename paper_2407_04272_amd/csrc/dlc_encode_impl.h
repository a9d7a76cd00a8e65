// The encode kernel for one chunk size S (DLC_S, defined by the including source file: one file per S keeps
// the compile times apart).
#include "dlc_codec_dev.h"

#define DLC_CAT2(a, b) a##b
#define DLC_CAT(a, b) DLC_CAT2(a, b)

// wavefronts per SIMD the register allocation aims at
#define DLC_ENC_WAVES(S) ((S) == 128 ? 3 : 4)

namespace dlc {

// ------------------------------------------------------------------------------------------------
// bit-packed encode.
//   walk 1: read the group's window indices from the symbol plane the histogram kernel has written (one byte per
//           element: 0..253 = symbol win_lo + index, 254 = escape, 255 = everything else), keep them in registers
//           four to a word, look up the code length of each in LDS and sum the chunk's bits.  Index 255 is rare (a
//           symbol outside the window, a position past the end of the table): its element is quantised again,
//           with the code from the full table.  Escapes are counted and where they are is remembered.
//   scan  : chunk word counts inside the wavefront; the wavefronts' totals (chunk words + two words per
//           escape) are joined per work-group, and the work-groups' totals across the grid by a single-pass
//           look-back (ordered work-group ids: a work-group only ever waits for work-groups that started
//           earlier)
//   walk 2: look up length and codeword of the kept indices (index 255: the element itself once more), join the
//           two codes of a pair, shift into a 64-bit accumulator, store whole words at the chunk's offset
//   escapes: their records (element index, raw bits; in increasing element index, behind the group's chunk words)
//           are written from the offsets kept in LDS during walk 1, up to 128 per group; a group with more walks
//           its elements once more in a rolled loop
// Keeping bytes instead of (length, codeword) entries halves the registers a wavefront holds between the walks,
// which doubles the wavefronts per SIMD: the kernel is bound by latency (global scan, table look-ups, stores),
// not by arithmetic.
// ------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) uint16_t lds_u16;
__device__ __forceinline__ uint32_t lds_read16(uint32_t addr, uint32_t byte_off) {
    return *reinterpret_cast<lds_u16*>(reinterpret_cast<__attribute__((address_space(3))) unsigned char*>(addr) + byte_off);
}


// (length << 12 | codeword) of the element at `off` of the group, quantised again; *is_escape says whether it is one
template <bool F16>
__device__ __forceinline__ uint32_t entry_of_element(const uint8_t* gbase, uint32_t off, const QParam& q, float Rf, int R,
                                                     const uint16_t* enc_t, uint32_t* is_escape) {
    float x;
    if constexpr (F16) x = __half2float(__ushort_as_half(reinterpret_cast<const unsigned short*>(gbase)[off]));
    else x = reinterpret_cast<const float*>(gbase)[off];
    const uint32_t sym = quant_symbol<F16>(x, q, Rf, R);
    *is_escape = sym == 0u ? 1u : 0u;
    return enc_t[sym];
}

__device__ __forceinline__ bool has_ff_byte(uint32_t m) {
    return ((m & 0xFFu) == 0xFFu) | ((m & 0xFF00u) == 0xFF00u) | ((m & 0xFF0000u) == 0xFF0000u) | (m >= 0xFF000000u);
}

template <int S, bool F16, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(DLC_ENC_WAVES(S))))
void k_encode(const void* payload, const uint8_t* sym_plane, Geom g, FixedLayout F, const QParam* qp, const uint16_t* enc,
              const TMeta* tmeta, Ctrl* ctrl, uint64_t* state, uint64_t epoch, uint8_t* out, uint64_t capacity, uint32_t bpt,
              uint32_t* word_start, uint32_t* word_end) {
    __shared__ __align__(16) uint16_t s_len[256], s_code[256];  // by window index; entry 255 is empty
    __shared__ uint32_t s_wg, s_tot[4], s_ct[4], s_excl, s_dead;
    // LDS staging per wavefront: room for a group of up to 4.7 bits per symbol, which is what four work-groups per
    // compute unit leave (with 4 bits a payload compressed 7 times no longer fitted and the kernel took twice as long)
    constexpr uint32_t kStageWords = 75u * (uint32_t)S / 8u;
    __shared__ __align__(16) uint32_t s_stage[4 * kStageWords];
    // escapes a wavefront remembers in LDS (their offsets in the group; the raw bits are read again when the records
    // are written); a group with more walks its elements again
    constexpr uint32_t kEncRecs = 128;
    __shared__ uint16_t s_recs[4 * kEncRecs];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid == 0) s_wg = atomicAdd(&ctrl->ticket, 1u);
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
    {
        // (index 254 is the escape, symbol 0; with row matching index 253 marks an element of a row that is stored as
        // a reference: no bits)
        const uint32_t c = win_lo + tid;
        const uint32_t e = tid == kWinEsc ? enc_t[0] : ((tid < win_bins(g.lz) && c < g.K) ? enc_t[c] : 0u);
        s_len[tid] = (uint16_t)(e >> 12);
        s_code[tid] = (uint16_t)(e & 0xFFFu);
    }
    __syncthreads();
    const uint32_t grp = b * 4 + wave;
    const bool active = grp < g.G;  // uniform over the wavefront; an idle wavefront only takes part in the barriers
    const uint32_t gid = tl * g.G + (active ? grp : 0u);  // group number inside the container
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t gstart = grp * (kW * (uint32_t)S);
    const uint8_t* gbase = tab + (size_t)gstart * g.es;
    const uint32_t rem = active ? g.n - gstart : 0u;
    // can index 255 occur in this group at all?  (an escape, a symbol outside the window, a ragged last group)
    const TMeta tm = tmeta[t];
    const bool plain = tm.n_outliers == 0u && tm.sym_lo >= win_lo && tm.sym_hi < win_lo + win_bins(g.lz) && rem >= kW * (uint32_t)S;
    const uint32_t a_len = (uint32_t)(uintptr_t)s_len, d_code = (uint32_t)(uintptr_t)s_code - a_len;

    uint32_t ix[S / 4];  // window indices, four to a word, in element order
    uint32_t bits = 0, my_esc = 0, nrec = 0;
    uint16_t* const recs = s_recs + wave * kEncRecs;
    if (active) {
        const uint32_t* plane = reinterpret_cast<const uint32_t*>(sym_plane + (size_t)t * plane_stride(g) + gstart);
        const bool ragged = rem < kW * (uint32_t)S;  // uniform: the table ends inside this group
#pragma clang loop unroll(full)
        for (int j = 0; j < S / 4; ++j) ix[j] = plane[(uint32_t)j * kW + lane];
        constexpr int kB1 = 4;  // words whose table reads are in flight together
#pragma clang loop unroll(full)
        for (int jb = 0; jb < S / 4; jb += kB1) {
            if (ragged) {  // whatever the plane holds past the end of the table does not count
#pragma clang loop unroll(full)
                for (int u = 0; u < kB1; ++u) {
                    const uint32_t off = lane * kV + (uint32_t)(jb + u) * (kW * kV);
                    uint32_t m = ix[jb + u];
#pragma clang loop unroll(full)
                    for (int v = 0; v < 4; ++v) m |= (off + (uint32_t)v < rem) ? 0u : (0xFFu << (8 * v));
                    ix[jb + u] = m;
                }
            }
            uint32_t l[kB1][4];
#pragma clang loop unroll(full)
            for (int u = 0; u < kB1; ++u)
#pragma clang loop unroll(full)
                for (int v = 0; v < 4; ++v) l[u][v] = lds_read16(a_len + (((ix[jb + u] >> (8 * v)) & 0xFFu) << 1), 0);
#pragma clang loop unroll(full)
            for (int u = 0; u < kB1; ++u) bits += l[u][0] + l[u][1] + l[u][2] + l[u][3];
            if (!plain) {  // uniform over the wavefront
#pragma clang loop unroll(full)
                for (int u = 0; u < kB1; ++u) {
                    const uint32_t m = ix[jb + u];
                    if (__ballot(has_ff_byte(m | 0x01010101u)) == 0ull) continue;  // nothing but window indices
                    uint32_t em = 0;  // which of the four are escapes (their bits are counted above: the table has their code)
#pragma clang loop unroll(full)
                    for (int v = 0; v < 4; ++v) em |= (((m >> (8 * v)) & 0xFFu) == kWinEsc ? 1u : 0u) << v;
                    my_esc += __popc(em);
                    if (__ballot(has_ff_byte(m)) != 0ull) {  // symbols outside the window
#pragma clang loop unroll(full)
                        for (int v = 0; v < 4; ++v) {
                            const uint32_t off = lane * kV + (uint32_t)(jb + u) * (kW * kV) + (uint32_t)v;
                            if (((m >> (8 * v)) & 0xFFu) == 0xFFu && off < rem) {
                                uint32_t esc;
                                bits += entry_of_element<F16>(gbase, off, q, Rf, (int)g.R, enc_t, &esc) >> 12;
                            }
                        }
                    }
                    // the records of these escapes, in element order (the walk meets the elements of a group in
                    // increasing index: turn, lane, position); kept in LDS while they fit
                    if (__ballot(em != 0u) != 0ull) {
                        const uint32_t cnt = __popc(em);
                        const uint32_t incl = wave_incl_scan(cnt, lane);
                        uint32_t r = nrec + incl - cnt;
#pragma clang loop unroll(full)
                        for (int v = 0; v < 4; ++v)
                            if ((em >> v) & 1u) {
                                if (r < kEncRecs) recs[r] = (uint16_t)(lane * kV + (uint32_t)(jb + u) * (kW * kV) + (uint32_t)v);
                                ++r;
                            }
                        nrec += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                    }
                }
            }
        }
    }
    const uint32_t n_esc = (plain || !active) ? 0u : wave_sum(my_esc);
    const uint32_t nw = (bits + 31u) >> 5;
    const uint32_t incl = wave_incl_scan(nw, lane);
    const uint32_t lane_off = incl - nw;
    const uint32_t chunk_total = __shfl(incl, 63, 64);
    const uint32_t total = chunk_total + 2u * n_esc;  // 0 for an idle wavefront

    // offsets: one scan record per work-group; the wavefronts' totals are joined through LDS.  The look-back over
    // the records of earlier work-groups is done by the first wavefront, a step at a time, in between its emit
    // work: walk 2 writes into an LDS staging buffer, which needs no global offset yet, and the words are copied to
    // their place (coalesced) once the offset is known.  A work-group with a group too large for the staging
    // buffer waits for its offset first and emits straight to memory.
    if (lane == 0) { s_tot[wave] = total; s_ct[wave] = chunk_total; }
    __syncthreads();
    const uint32_t wg_total = s_tot[0] + s_tot[1] + s_tot[2] + s_tot[3];
    const bool staged = max(max(s_ct[0], s_ct[1]), max(s_ct[2], s_ct[3])) <= kStageWords;  // uniform over the work-group
    LookBack L;
    lb_init(L, wg, dom0);
    if (wave == 0) lb_publish_aggregate(state, epoch, wg, wg_total, lane, dom0);
    if (!staged) {
        if (wave == 0) {
            lb_finish(L, state, epoch, wg, wg_total, lane, ctrl);
            if (lane == 0) { s_excl = L.excl; s_dead = L.failed ? 1u : 0u; }
        }
        __syncthreads();
    }
    uint32_t excl = 0;
    bool dead = false;  // nothing may be written to the container
    if (!staged) {
        dead = s_dead != 0u;
        excl = s_excl;
        for (uint32_t k = 0; k < wave; ++k) excl += s_tot[k];
        if (F.off_payload + 4ull * ((uint64_t)excl + total) > capacity) {
            if (active && !dead && lane == 0) { set_status(ctrl, DLC_ECAPACITY); atomicOr(&ctrl->abort, kAbortCapacity); }
            dead = true;
        }
    }
    uint32_t* const stage = s_stage + wave * kStageWords;
    if (active && !(dead && !staged)) {
        uint32_t* p = staged ? stage + lane_off : reinterpret_cast<uint32_t*>(out + F.off_payload) + excl + lane_off;
        uint64_t acc = 0;
        uint32_t nb = 0;
        constexpr int kB2 = 2;  // words of indices whose table reads are in flight together
#pragma clang loop unroll(full)
        for (int jb = 0; jb < S / 4; jb += kB2) {
            if (staged && wave == 0 && !L.done && (jb % 8) == 0) {  // uniform: one look-back step per eight words
                if (L.pending) (void)lb_consume(L, epoch, lane);
                if (!L.done) lb_issue(L, state, epoch, lane);
            }
            uint32_t l[kB2][4], c[kB2][4];
#pragma clang loop unroll(full)
            for (int u = 0; u < kB2; ++u) {
                uint32_t m = ix[jb + u];
                asm volatile("" : "+v"(m));  // unpack here, not where the word was made
#pragma clang loop unroll(full)
                for (int v = 0; v < 4; ++v) {
                    const uint32_t a = a_len + (((m >> (8 * v)) & 0xFFu) << 1);
                    l[u][v] = lds_read16(a, 0);
                    c[u][v] = lds_read16(a, d_code);
                }
                if (!plain && __ballot(has_ff_byte(m)) != 0ull) {  // uniform over the wavefront
#pragma clang loop unroll(full)
                    for (int v = 0; v < 4; ++v) {
                        const uint32_t off = lane * kV + (uint32_t)(jb + u) * (kW * kV) + (uint32_t)v;
                        if (((m >> (8 * v)) & 0xFFu) == 0xFFu && off < rem) {
                            uint32_t esc;
                            const uint32_t e = entry_of_element<F16>(gbase, off, q, Rf, (int)g.R, enc_t, &esc);
                            l[u][v] = e >> 12;
                            c[u][v] = e & 0xFFFu;
                        }
                    }
                }
            }
#pragma clang loop unroll(full)
            for (int u = 0; u < kB2; ++u)
#pragma clang loop unroll(full)
                for (int h = 0; h < 2; ++h) {
                    const uint32_t len = l[u][2 * h] + l[u][2 * h + 1];  // a pair: at most 24 bits
                    acc = (acc << len) | ((c[u][2 * h] << l[u][2 * h + 1]) | c[u][2 * h + 1]);
                    nb += len;
                    if (nb >= 32u) {
                        nb -= 32u;
                        *p++ = (uint32_t)(acc >> nb);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (nb) *p = (uint32_t)(acc << (32u - nb));
    }
    if (staged) {
        if (wave == 0) {
            lb_finish(L, state, epoch, wg, wg_total, lane, ctrl);
            if (lane == 0) { s_excl = L.excl; s_dead = L.failed ? 1u : 0u; }
        }
        __syncthreads();  // also: the staging buffers are complete
        dead = s_dead != 0u;
        excl = s_excl;
        for (uint32_t k = 0; k < wave; ++k) excl += s_tot[k];
        if (F.off_payload + 4ull * ((uint64_t)excl + total) > capacity) {
            if (active && !dead && lane == 0) { set_status(ctrl, DLC_ECAPACITY); atomicOr(&ctrl->abort, kAbortCapacity); }
            dead = true;
        }
    }
    if (!active) return;
    if (lane == 0) {
        if (grp == 0) word_start[t] = excl;
        if (grp == g.G - 1) word_end[t] = excl + total;
    }
    if (dead) return;
    out[F.off_chunk + (uint64_t)gid * kW + lane] = (uint8_t)nw;
    if (lane == 0) reinterpret_cast<uint32_t*>(out + F.off_group)[gid] = excl;
    uint32_t* gw = reinterpret_cast<uint32_t*>(out + F.off_payload) + excl;
    if (staged)
        for (uint32_t k = lane; k < chunk_total; k += 64) gw[k] = stage[k];
    if (n_esc != 0u) {  // uniform over the wavefront
        uint32_t* rec = gw + chunk_total;
        if (n_esc <= kEncRecs) {  // the records were kept on the way
            for (uint32_t k = lane; k < n_esc; k += 64) {
                const uint32_t off = recs[k];
                rec[2u * k] = gstart + off;
                if constexpr (F16) rec[2u * k + 1] = reinterpret_cast<const uint16_t*>(gbase)[off];
                else rec[2u * k + 1] = reinterpret_cast<const uint32_t*>(gbase)[off];
            }
        } else {
            emit_escapes<S, F16, VEC>(rec, lane, gbase, reinterpret_cast<const uint32_t*>(sym_plane + (size_t)t * plane_stride(g) + gstart),
                                      gstart, rem);
        }
    }
}

void DLC_CAT(launch_encode_, DLC_S)(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch,
                                    uint8_t* out, uint64_t capacity, uint32_t bpt, hipStream_t s) {
    constexpr int S = DLC_S;
    dim3 grid(g.T * bpt), block(256);
    const size_t sm = 0;
    const bool f16 = g.dtype == DLC_F16;
#define DLC_ENC(FF, V)                                                                                          \
    hipLaunchKernelGGL((k_encode<S, FF, V>), grid, block, sm, s, payload, w.sym_plane, g, F, w.qp, w.enc, w.tmeta, w.ctrl, w.state, epoch, \
                       out, capacity, bpt, w.word_start, w.word_end)
    if (f16) { if (g.vec) DLC_ENC(true, true); else DLC_ENC(true, false); }
    else { if (g.vec) DLC_ENC(false, true); else DLC_ENC(false, false); }
#undef DLC_ENC
}

}  // namespace dlc
