// The fused compress kernel for one chunk size S (DLC_S, defined by the including source file).
#include "dlc_codec_dev.h"

#define DLC_CAT2(a, b) a##b
#define DLC_CAT(a, b) DLC_CAT2(a, b)

// phase time stamps of one item, for micro-benchmarks only (compiled out of the library)
#ifdef DLC_EXP_STAMPS
__device__ long long g_fstamp[32];
#define DLC_FSTAMP(i) do { if (item == DLC_EXP_STAMPS && threadIdx.x == 0) g_fstamp[i] = wall_clock64(); } while (0)
extern "C" void dlc_debug_stamps(long long* out) { (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_fstamp), sizeof(g_fstamp)); }
#else
#define DLC_FSTAMP(i)
#endif

#ifndef DLC_FUSED_WAVES  // wavefronts per SIMD the register allocation aims at
#define DLC_FUSED_WAVES(S) ((S) == 256 ? 2 : ((S) == 128 ? 3 : 4))
#endif

namespace dlc {

// ------------------------------------------------------------------------------------------------
// Fused compress: one persistent kernel that reads every element once.
//   A work-group takes items in ticket order; an item is four consecutive groups of one table (one per
//   wavefront).
//   phase A  load, quantise, count into the work-group's LDS histogram, keep the symbols in registers
//            (two per register, as LDS addresses of their code-table entries); add the histogram to the
//            table's global one; the last of the table's items to arrive builds the table's codebook and
//            publishes it
//   phase B  wait for the codebook, replace each kept pair of symbols by one (length, bits) entry, then
//            chunk sizes, look-back over groups, emit, escapes
//   Progress: a work-group waits only for items with smaller tickets (look-back) or for the items of its own
//   table (codebook); tickets go to running work-groups in increasing order, so once at least `bpt`
//   work-groups run, the table of the smallest unfinished ticket completes.  The host launches this kernel
//   only when the resident grid is at least twice that.  Every wait is bounded.
//   No fences anywhere (a device-scope fence writes back and invalidates the whole L2 of the die): everything
//   other work-groups read goes through device-scope atomics, and a thread waits for its own to be
//   acknowledged before the barrier that precedes the next signal.
// ------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(3))) uint16_t lds_u16;
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void lds_count(uint32_t addr) {
    __hip_atomic_fetch_add(reinterpret_cast<lds_u32*>(addr), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ uint32_t lds_read16(uint32_t addr, uint32_t byte_off) {
    return *reinterpret_cast<lds_u16*>(reinterpret_cast<__attribute__((address_space(3))) unsigned char*>(addr) + byte_off);
}

// constants of phase A
struct FusedA {
    int ubias;           // window index of bin 0: a coded element with bin r has window index r + ubias
    uint32_t u_esc;      // window index that stands for the escape (maps to table entry K)
    uint32_t u_inv;      // ... for a position past the end of the table (maps to table entry 0)
    uint32_t win_bins;   // rows of the window; row win_bins counts everything outside
    uint32_t lanebase;   // LDS address of this lane's copy of window row 0
    uint32_t trash;      // LDS address of this lane's scratch word
    uint32_t pkc;        // both halves: 2*win_lo + LDS address of the length table
};

// FULL: every position of the group is inside the table (no masking at all)
template <int S, bool F16, bool VEC, bool FULL>
__device__ __forceinline__ void fused_symbols(const uint8_t* gbase, uint32_t rem, uint32_t lane, const QParam& q, float Rf,
                                              const FusedA& A, uint32_t (&pk)[S / 2]) {
    constexpr int kBlk = 8;
#pragma clang loop unroll(full)
    for (int jb = 0; jb < S / 4; jb += kBlk) {
        float x[kBlk][4];
        uint32_t raw[kBlk][4];
        uint32_t valid[kBlk];
#pragma clang loop unroll(full)
        for (int u = 0; u < kBlk; ++u)
            valid[u] = load4<F16, VEC>(gbase, lane * kV + (uint32_t)(jb + u) * (kW * kV), FULL ? 0xFFFFFFFFu : rem, x[u],
                                       raw[u]);
#pragma clang loop unroll(full)
        for (int u = 0; u < kBlk; ++u) {
            uint32_t ui[4];
#pragma clang loop unroll(full)
            for (int v = 0; v < 4; ++v) {
                // the quantiser (same arithmetic as quant_symbol), result as a window index
                const float xv = x[u][v];
                const float r = __builtin_rintf(xv * q.inv);
                float xh = r * q.ebx2;
                if constexpr (F16) xh = __half2float(half_rne(xh));
                const float d = xv - xh;
                const bool ok = (__builtin_fabsf(r) < Rf) & (__builtin_fabsf(d) <= q.eb);  // no short circuit: no branches
                uint32_t w = ok ? (uint32_t)((int)r + A.ubias) : A.u_esc;
                uint32_t addr = min(w, A.win_bins) * (kFusedCopies * 4u) + A.lanebase;
                if constexpr (!FULL) {
                    const bool in = (valid[u] >> v) & 1u;
                    addr = in ? addr : A.trash;
                    w = in ? w : A.u_inv;
                }
                lds_count(addr);
                ui[v] = w;
            }
            // low halves of two indices in one word, then index -> LDS address of the table entry, both halves at once
            uint32_t w0 = __builtin_amdgcn_perm(ui[1], ui[0], 0x05040100u), w1 = __builtin_amdgcn_perm(ui[3], ui[2], 0x05040100u);
            const us2 c = __builtin_bit_cast(us2, A.pkc);
            w0 = __builtin_bit_cast(uint32_t, (us2)(__builtin_bit_cast(us2, w0) * (us2)(2) + c));
            w1 = __builtin_bit_cast(uint32_t, (us2)(__builtin_bit_cast(us2, w1) * (us2)(2) + c));
            asm volatile("" : "+v"(w0), "+v"(w1));  // keep the symbols packed
            pk[2 * (jb + u)] = w0;
            pk[2 * (jb + u) + 1] = w1;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The codebook builder as a real call: it runs once per table, and inlined its registers would come on top of the
// symbols every wavefront keeps across it.
__device__ __noinline__ void fused_codebook(const Geom& g, uint32_t* hist_t, uint32_t* hist_view_t, uint16_t* enc_t,
                                            uint8_t* lens_t, TMeta* tmeta_t, unsigned char* smem, CodebookShared& sh,
                                            uint32_t tid) {
    codebook_build(g, hist_t, hist_view_t, enc_t, lens_t, tmeta_t, smem, sh, tid);
}

// what a work-group keeps about an item between its two phases
struct FusedItem {
    uint32_t t, grp, gid, gstart, rem, n_esc;
    bool active;  // this wavefront has a group (uniform over the wavefront)
    const uint8_t* gbase;
    QParam q;
};

// everything of the kernel that does not change from item to item
struct FusedEnv {
    Geom g;
    FixedLayout F;
    const void* payload;
    const QParam* qp;
    uint32_t *hist, *hist_view;
    uint16_t* enc;
    uint8_t* lens;
    TMeta* tmeta;
    Ctrl* ctrl;
    uint32_t* arrive;
    uint64_t *ready, *state;
    uint64_t epoch, capacity;
    uint8_t* out;
    uint32_t bpt;
    uint32_t *word_start, *word_end;
    // LDS
    unsigned char* region;
    uint32_t *lh, *ovf;
    uint16_t *tab_len, *tab_code;
    uint32_t win_bins, win_lo, n_words, tab0;
    float Rf;
};

// phase A of one item; ends with the item's counts added to the table's histogram and, if this was the last
// item of the table, with the table's codebook published.  Called by all threads (has barriers).
template <int S, bool F16, bool VEC>
__device__ __forceinline__ void fused_phase_a(const FusedEnv& E, const FusedA& A, uint32_t item, FusedItem& I,
                                              uint32_t (&pk)[S / 2], CodebookShared& sh, uint32_t* s_last, uint32_t tid,
                                              uint32_t lane, uint32_t wave) {
    const Geom& g = E.g;
    I.t = item / E.bpt;
    const uint32_t b = item % E.bpt;
    DLC_FSTAMP(0);
    {
        uint4* z = reinterpret_cast<uint4*>(E.region);
        for (uint32_t k = tid; k < (E.n_words + 3u) / 4u; k += 256) z[k] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    I.grp = b * 4 + wave;
    I.active = I.grp < g.G;
    I.gid = I.t * g.G + I.grp;
    I.q = E.qp[I.t];
    const uint8_t* tab = static_cast<const uint8_t*>(E.payload) + (size_t)I.t * g.n * g.es;
    I.gstart = I.grp * (kW * (uint32_t)S);
    I.gbase = tab + (size_t)I.gstart * g.es;
    I.rem = I.active ? g.n - I.gstart : 0u;
    DLC_FSTAMP(1);
    if (I.active) {
        if (I.rem >= kW * (uint32_t)S) fused_symbols<S, F16, VEC, true>(I.gbase, I.rem, lane, I.q, E.Rf, A, pk);
        else fused_symbols<S, F16, VEC, false>(I.gbase, I.rem, lane, I.q, E.Rf, A, pk);
    }
    DLC_FSTAMP(2);
    __syncthreads();
    DLC_FSTAMP(3);
    // anything outside the window (escapes included) was only counted as such: if there is any, walk the kept
    // symbols once more for the exact counts and for the group's number of escapes
    I.n_esc = 0;
    {
        const uint32_t o = lane < kFusedCopies ? E.lh[E.win_bins * kFusedCopies + lane] : 0u;
        if (__ballot(o != 0u) != 0ull) {  // same answer in every wavefront of the work-group
            if (I.active) {
                uint32_t n_esc = 0;
#pragma clang loop unroll(full)
                for (int i = 0; i < S / 2; ++i) {
                    const uint32_t w = pk[i];
#pragma clang loop unroll(full)
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t c2 = ((h ? (w >> 16) : (w & 0xFFFFu)) - E.tab0) & 0xFFFFu;  // twice the symbol
                        const bool esc = c2 == 2u * g.K;
                        n_esc += (uint32_t)__popcll(__ballot(esc));
                        if (!esc && c2 != 0u && (c2 >> 1) - E.win_lo >= E.win_bins) atomicAdd(&E.ovf[c2 >> 1], 1u);
                    }
                }
                if (lane == 0 && n_esc) atomicAdd(&E.ovf[0], n_esc);
                I.n_esc = n_esc;
            }
            __syncthreads();
        }
    }
    for (uint32_t k = tid; k < g.K; k += 256) {
        uint32_t s = E.ovf[k];
        const uint32_t w = k - E.win_lo;
        if (w < E.win_bins) {
            const uint32_t* row = E.lh + w * kFusedCopies;
            for (uint32_t c = 0; c < kFusedCopies; ++c) s += row[(c + tid) & (kFusedCopies - 1u)];
        }
        if (s) atomicAdd(&E.hist[(size_t)I.t * g.K + k], s);
    }
    DLC_FSTAMP(4);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    DLC_FSTAMP(5);
    if (tid == 0)
        *s_last = (__hip_atomic_fetch_add(&E.arrive[I.t], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == E.bpt) ? 1u : 0u;
    __syncthreads();
    if (*s_last) {  // uniform: every item of the table has added its counts
        const size_t o = (size_t)I.t * g.K;
        fused_codebook(g, E.hist + o, E.hist_view + o, E.enc + o, E.lens + o, E.tmeta + I.t, E.region, sh, tid);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            __hip_atomic_store(&E.arrive[I.t], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next call
            __hip_atomic_store(&E.ready[I.t], E.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    DLC_FSTAMP(6);
}

// phase B of one item: waits for the table's codebook.  Called by all threads (has barriers).
template <int S, bool F16, bool VEC>
__device__ __forceinline__ void fused_phase_b(const FusedEnv& E, const FusedItem& I, uint32_t (&pk)[S / 2], uint32_t* s_go,
                                              uint32_t* s_tot, uint32_t tid, uint32_t lane, uint32_t wave) {
    const Geom& g = E.g;
#ifdef DLC_EXP_STAMPS
    const uint32_t item = I.t * E.bpt + I.grp / 4;
#endif
    DLC_FSTAMP(7);
    if (tid == 0) {
        uint32_t spins = 0, go = 1;
        while (__hip_atomic_load(&E.ready[I.t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != E.epoch) {
            if (++spins > kSpinLimit) {  // never expected; the bound only guarantees termination
                set_status(E.ctrl, DLC_ESTATE);
                atomicOr(&E.ctrl->abort, kAbortInternal);
                go = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        *s_go = go;
    }
    __syncthreads();
    DLC_FSTAMP(8);
    bool dead = *s_go == 0u;
    for (uint32_t k = tid; k <= g.K; k += 256) {
        // entry 0: a position past the end (no bits); entry K: the escape, which is symbol 0 of the codebook
        const uint32_t src = k == g.K ? 0u : k;
        uint32_t e = __hip_atomic_load(&E.enc[(size_t)I.t * g.K + src], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (k == 0) e = 0;
        E.tab_len[k] = (uint16_t)(e >> 12);
        E.tab_code[k] = (uint16_t)(e & 0xFFFu);
    }
    __syncthreads();
    DLC_FSTAMP(9);
    uint32_t bits = 0;
    if (I.active) {
        constexpr int kB = 8;  // pairs whose table reads are in flight together
#pragma clang loop unroll(full)
        for (int ib = 0; ib < S / 2; ib += kB) {
            uint32_t l0[kB], c0[kB], l1[kB], c1[kB];
#pragma clang loop unroll(full)
            for (int u = 0; u < kB; ++u) {
                const uint32_t w = pk[ib + u];
                const uint32_t a0 = w & 0xFFFFu, a1 = w >> 16;
                l0[u] = lds_read16(a0, 0); c0[u] = lds_read16(a0, kFusedTab);
                l1[u] = lds_read16(a1, 0); c1[u] = lds_read16(a1, kFusedTab);
            }
#pragma clang loop unroll(full)
            for (int u = 0; u < kB; ++u) {
                const uint32_t len = l0[u] + l1[u];
                uint32_t w2 = (len << 24) | (c0[u] << l1[u]) | c1[u];  // at most 24 bits of code
                asm volatile("" : "+v"(w2));
                pk[ib + u] = w2;
                bits += len;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        DLC_FSTAMP(10);
    }
    const uint32_t nw = (bits + 31u) >> 5;
    const uint32_t incl = wave_incl_scan(nw, lane);
    const uint32_t lane_off = incl - nw;
    const uint32_t chunk_total = __shfl(incl, 63, 64);
    const uint32_t total = chunk_total + 2u * I.n_esc;  // 0 for an idle wavefront
    // offsets: one scan record per item; the wavefronts' totals are joined through LDS
    if (lane == 0) s_tot[wave] = total;
    __syncthreads();
    if (wave == 0) {
        const uint32_t e = wg_scan(E.state, E.epoch, I.t * E.bpt + I.grp / 4u, s_tot[0] + s_tot[1] + s_tot[2] + s_tot[3], lane,
                                   E.ctrl, &dead);
        if (lane == 0) { s_tot[4] = e; s_tot[5] = dead ? 1u : 0u; }
    }
    __syncthreads();
    if (I.active) {
        dead = s_tot[5] != 0u;
        uint32_t excl = s_tot[4];
        for (uint32_t k = 0; k < wave; ++k) excl += s_tot[k];
        DLC_FSTAMP(11);
        if (E.F.off_payload + 4ull * ((uint64_t)excl + total) > E.capacity) {
            if (!dead && lane == 0) { set_status(E.ctrl, DLC_ECAPACITY); atomicOr(&E.ctrl->abort, kAbortCapacity); }
            dead = true;
        }
        if (lane == 0) {
            if (I.grp == 0) E.word_start[I.t] = excl;
            if (I.grp == g.G - 1) E.word_end[I.t] = excl + total;
        }
        if (!dead) {
            E.out[E.F.off_chunk + (uint64_t)I.gid * kW + lane] = (uint8_t)nw;
            if (lane == 0) reinterpret_cast<uint32_t*>(E.out + E.F.off_group)[I.gid] = excl;
            uint32_t* gw = reinterpret_cast<uint32_t*>(E.out + E.F.off_payload) + excl;
            uint32_t* p = gw + lane_off;
            uint64_t acc = 0;
            uint32_t nb = 0;
#pragma clang loop unroll(full)
            for (int i = 0; i < S / 2; ++i) {
                uint32_t w = pk[i];
                asm volatile("" : "+v"(w));  // unpack here, not where the entry was made
                const uint32_t len = w >> 24;
                acc = (acc << len) | (w & 0xFFFFFFu);
                nb += len;
                if (nb >= 32u) {
                    nb -= 32u;
                    *p++ = (uint32_t)(acc >> nb);
                }
                if ((i & 3) == 3) __builtin_amdgcn_sched_barrier(0);
            }
            if (nb) *p = (uint32_t)(acc << (32u - nb));
            if (I.n_esc != 0u)  // uniform over the wavefront
                emit_escapes<S, F16, VEC>(gw + chunk_total, lane, I.gbase, I.gstart, I.rem, I.q, E.Rf, (int)g.R);
        }
        DLC_FSTAMP(12);
    }
}

template <int S, bool F16, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(DLC_FUSED_WAVES(S))))
void k_fused(const void* payload, Geom g, FixedLayout F, const QParam* qp, uint32_t* hist, uint32_t* hist_view,
             uint16_t* enc, uint8_t* lens, TMeta* tmeta, Ctrl* ctrl, uint32_t* arrive, uint64_t* ready, uint64_t* state,
             uint64_t epoch, uint8_t* out, uint64_t capacity, uint32_t bpt, uint32_t n_items, uint32_t* word_start,
             uint32_t* word_end) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ CodebookShared sh;
    __shared__ uint32_t s_item, s_last, s_go, s_tot[6];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;  // LDS address of the dynamic part
    FusedEnv E;
    E.g = g; E.F = F; E.payload = payload; E.qp = qp; E.hist = hist; E.hist_view = hist_view; E.enc = enc; E.lens = lens;
    E.tmeta = tmeta; E.ctrl = ctrl; E.arrive = arrive; E.ready = ready; E.state = state; E.epoch = epoch;
    E.capacity = capacity; E.out = out; E.bpt = bpt; E.word_start = word_start; E.word_end = word_end;
    E.tab_len = reinterpret_cast<uint16_t*>(smem);
    E.tab_code = reinterpret_cast<uint16_t*>(smem + kFusedTab);
    E.region = smem + 2 * kFusedTab;
    E.lh = reinterpret_cast<uint32_t*>(E.region);
    E.win_bins = hist_win_bins(g.K);
    E.win_lo = g.R - E.win_bins / 2u;
    E.n_words = (E.win_bins + 1u) * kFusedCopies + g.K + kW;
    E.ovf = E.lh + (E.win_bins + 1u) * kFusedCopies;
    E.tab0 = lds0 & 0xFFFFu;  // what an address kept in pk[] has on top of twice the symbol
    E.Rf = (float)g.R;
    FusedA A;
    A.ubias = (int)(E.win_bins / 2u);
    A.u_esc = g.K - E.win_lo;
    A.u_inv = 0u - E.win_lo;
    A.win_bins = E.win_bins;
    A.lanebase = lds0 + 2u * kFusedTab + (lane & (kFusedCopies - 1u)) * 4u;
    A.trash = lds0 + 2u * kFusedTab + ((E.win_bins + 1u) * kFusedCopies + g.K + lane) * 4u;
    {
        const uint32_t h = (2u * E.win_lo + lds0) & 0xFFFFu;
        A.pkc = h | (h << 16);
    }

    {
        uint32_t pk[S / 2];
        FusedItem I;
        for (;;) {
            if (tid == 0) s_item = atomicAdd(&ctrl->ticket, 1u);
            __syncthreads();  // also: the previous item is done with the LDS
            const uint32_t item = __builtin_amdgcn_readfirstlane(s_item);
            if (item >= n_items) break;
            fused_phase_a<S, F16, VEC>(E, A, item, I, pk, sh, &s_last, tid, lane, wave);
            fused_phase_b<S, F16, VEC>(E, I, pk, &s_go, s_tot, tid, lane, wave);
        }
    }
}

// the instantiation for a geometry
const void* DLC_CAT(fused_kernel_, DLC_S)(const Geom& g) {
    constexpr int S = DLC_S;
#ifdef DLC_EXP_ONE_INST  // micro-benchmarks: one instantiation keeps the build short
    return reinterpret_cast<const void*>(k_fused<S, false, true>);
#else
    if (g.dtype == DLC_F16)
        return g.vec ? reinterpret_cast<const void*>(k_fused<S, true, true>) : reinterpret_cast<const void*>(k_fused<S, true, false>);
    return g.vec ? reinterpret_cast<const void*>(k_fused<S, false, true>) : reinterpret_cast<const void*>(k_fused<S, false, false>);
#endif
}

}  // namespace dlc
