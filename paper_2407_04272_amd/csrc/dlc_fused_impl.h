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

namespace dlc {

// ------------------------------------------------------------------------------------------------
// Fused compress: one persistent kernel that reads every element once.
//   A work-group takes items in ticket order; an item is four consecutive groups of one table (one per
//   wavefront).
//   phase A  load, quantise, count into the work-group's LDS histogram, keep the symbols in registers
//            (two per register, as byte offsets into the LDS code table); add the histogram to the table's
//            global one; the last of the table's items to arrive builds the table's codebook and publishes it
//   phase B  wait for the codebook, replace the kept symbols by their (length, codeword) entries, then as
//            in the encode kernel: chunk sizes, look-back over groups, emit, escapes
//   Progress: a work-group waits only for items with smaller tickets (look-back) or for the items of its own
//   table (codebook); tickets go to running work-groups in increasing order, so once at least `bpt`
//   work-groups run, the table of the smallest unfinished ticket completes.  The host launches this kernel
//   only when the resident grid is at least twice that.  Every wait is bounded.
// ------------------------------------------------------------------------------------------------
template <int S, bool F16, bool VEC>
__device__ __forceinline__ void fused_symbols(const uint8_t* gbase, uint32_t rem, uint32_t lane, const QParam& q, float Rf,
                                              int R, uint32_t K, uint32_t* lh, const HistLds& H, uint32_t (&pk)[S / 2]) {
    const uint32_t copy4 = (lane & (kHistCopies - 1u)) * 4u;
    constexpr int kBlk = 8;
#pragma clang loop unroll(full)
    for (int jb = 0; jb < S / 4; jb += kBlk) {
        float x[kBlk][4];
        uint32_t raw[kBlk][4];
        uint32_t valid[kBlk];
#pragma clang loop unroll(full)
        for (int u = 0; u < kBlk; ++u)
            valid[u] = load4<F16, VEC>(gbase, lane * kV + (uint32_t)(jb + u) * (kW * kV), rem, x[u], raw[u]);
#pragma clang loop unroll(full)
        for (int u = 0; u < kBlk; ++u) {
            uint32_t s2[4];
#pragma clang loop unroll(full)
            for (int v = 0; v < 4; ++v) {
                const uint32_t c = quant_symbol<F16>(x[u][v], q, Rf, R);
                const bool ok = (valid[u] >> v) & 1u;
                const uint32_t w = c - H.win_lo;  // wraps for symbols below the window
                uint32_t byte = w < H.win_bins ? w * (kHistCopies * 4u) + copy4 : H.ovf_byte + c * 4u;
                byte = ok ? byte : H.trash_byte;
                atomicAdd(reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(lh) + byte), 1u);
                s2[v] = ok ? c * 2u : K * 2u;  // entry K of the code table is empty: a position past the end adds no bits
            }
            uint32_t w0 = s2[0] | (s2[1] << 16), w1 = s2[2] | (s2[3] << 16);
            asm volatile("" : "+v"(w0), "+v"(w1));  // keep the symbols packed
            pk[2 * (jb + u)] = w0;
            pk[2 * (jb + u) + 1] = w1;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int S, bool F16, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(S == 256 ? 2 : (S == 128 ? 3 : 5))))
void k_fused(const void* payload, Geom g, FixedLayout F, const QParam* qp, uint32_t* hist, uint32_t* hist_view,
             uint16_t* enc, uint8_t* lens, TMeta* tmeta, Ctrl* ctrl, uint32_t* arrive, uint64_t* ready, uint64_t* state,
             uint64_t epoch, uint8_t* out, uint64_t capacity, uint32_t bpt, uint32_t n_items, uint32_t* word_start,
             uint32_t* word_end) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ CodebookShared sh;
    __shared__ uint32_t s_item, s_last, s_go;
    uint32_t* lh = reinterpret_cast<uint32_t*>(smem);
    const unsigned char* s_enc = smem + fused_region0(g.K);
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    HistLds H;
    H.win_bins = hist_win_bins(g.K);
    H.win_lo = g.R - H.win_bins / 2u;
    const uint32_t n_words = H.win_bins * kHistCopies + g.K + kW;
    H.ovf_byte = H.win_bins * kHistCopies * 4u;
    H.trash_byte = (H.win_bins * kHistCopies + g.K + lane) * 4u;
    const uint32_t* ovf = lh + H.win_bins * kHistCopies;
    const float Rf = (float)g.R;

    for (;;) {
        if (tid == 0) s_item = atomicAdd(&ctrl->ticket, 1u);
        __syncthreads();  // also: the previous item is done with the LDS
        const uint32_t item = __builtin_amdgcn_readfirstlane(s_item);
        if (item >= n_items) break;
        const uint32_t t = item / bpt, b = item % bpt;
        DLC_FSTAMP(0);
        for (uint32_t k = tid; k < n_words; k += 256) lh[k] = 0;
        __syncthreads();
        const uint32_t grp = b * 4 + wave;
        const bool active = grp < g.G;  // uniform over the wavefront
        const uint32_t gid = t * g.G + grp;
        const QParam q = qp[t];
        const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
        const uint32_t gstart = grp * (kW * (uint32_t)S);
        const uint8_t* gbase = tab + (size_t)gstart * g.es;
        const uint32_t rem = active ? g.n - gstart : 0u;

        // ---- phase A
        uint32_t pk[S / 2];
        DLC_FSTAMP(1);
        if (active) fused_symbols<S, F16, VEC>(gbase, rem, lane, q, Rf, (int)g.R, g.K, lh, H, pk);
        DLC_FSTAMP(2);
        __syncthreads();
        DLC_FSTAMP(3);
        // escapes are symbol 0, which lies outside the window: the work-group's count is one word
        uint32_t n_esc = 0;
        if (active && ovf[0] != 0u) {
#pragma clang loop unroll(full)
            for (int i = 0; i < S / 2; ++i) {
                const uint32_t w = pk[i];
                n_esc += (uint32_t)__popcll(__ballot((w & 0xFFFFu) == 0u)) + (uint32_t)__popcll(__ballot((w >> 16) == 0u));
            }
        }
        for (uint32_t k = tid; k < g.K; k += 256) {
            uint32_t s = ovf[k];
            const uint32_t w = k - H.win_lo;
            if (w < H.win_bins) {
                const uint32_t* row = lh + w * kHistCopies;
                for (uint32_t c = 0; c < kHistCopies; ++c) s += row[(c + tid) & (kHistCopies - 1u)];
            }
            if (s) atomicAdd(&hist[(size_t)t * g.K + k], s);
        }
        DLC_FSTAMP(4);
        // No fences anywhere in this kernel (a device-scope fence writes back and invalidates the whole L2 of the
        // die): everything other work-groups read goes through device-scope atomics, and a thread waits for its
        // own to be acknowledged before the barrier that precedes the next signal.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        DLC_FSTAMP(5);
        if (tid == 0)
            s_last = (__hip_atomic_fetch_add(&arrive[t], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == bpt) ? 1u : 0u;
        __syncthreads();
        if (s_last) {  // uniform: every item of the table has added its counts
            codebook_build(g, hist + (size_t)t * g.K, hist_view + (size_t)t * g.K, enc + (size_t)t * g.K,
                           lens + (size_t)t * g.K, tmeta + t, smem, sh, tid);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (tid == 0) {
                __hip_atomic_store(&arrive[t], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next call
                __hip_atomic_store(&ready[t], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        DLC_FSTAMP(6);
        // ---- wait for the table's codebook
        if (tid == 0) {
            uint32_t spins = 0, go = 1;
            while (__hip_atomic_load(&ready[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
                if (++spins > kSpinLimit) {  // never expected; the bound only guarantees termination
                    set_status(ctrl, DLC_ESTATE);
                    ctrl->abort = 1;
                    go = 0;
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
            s_go = go;
        }
        __syncthreads();
        DLC_FSTAMP(7);
        bool dead = s_go == 0u;
        {
            uint16_t* se = reinterpret_cast<uint16_t*>(smem + fused_region0(g.K));
            for (uint32_t k = tid; k < g.K; k += 256)
                se[k] = __hip_atomic_load(&enc[(size_t)t * g.K + k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (tid == 0) se[g.K] = 0;
        }
        __syncthreads();

        // ---- phase B
        DLC_FSTAMP(8);
        if (active) {
            uint32_t bits = 0;
#pragma clang loop unroll(full)
            for (int i = 0; i < S / 2; ++i) {
                const uint32_t w = pk[i];
                const uint32_t e0 = *reinterpret_cast<const uint16_t*>(s_enc + (w & 0xFFFFu));
                const uint32_t e1 = *reinterpret_cast<const uint16_t*>(s_enc + (w >> 16));
                uint32_t w2 = e0 | (e1 << 16);
                asm volatile("" : "+v"(w2));
                pk[i] = w2;
                bits += ((w2 >> 12) & 0xFu) + (w2 >> 28);
            }
            DLC_FSTAMP(9);
            const uint32_t nw = (bits + 31u) >> 5;
            const uint32_t incl = wave_incl_scan(nw, lane);
            const uint32_t lane_off = incl - nw;
            const uint32_t chunk_total = __shfl(incl, 63, 64);
            const uint32_t total = chunk_total + 2u * n_esc;
            const uint32_t excl = group_scan(state, epoch, gid, total, lane, ctrl, &dead);
            DLC_FSTAMP(10);
            if (F.off_payload + 4ull * ((uint64_t)excl + total) > capacity) {
                if (!dead && lane == 0) { set_status(ctrl, DLC_ECAPACITY); ctrl->abort = 1; }
                dead = true;
            }
            if (lane == 0) {
                if (grp == 0) word_start[t] = excl;
                if (grp == g.G - 1) word_end[t] = excl + total;
            }
            if (!dead)
                emit_group<S, F16, VEC>(pk, nw, lane_off, excl, chunk_total, n_esc, gid, lane, gbase, gstart, rem, q, Rf,
                                        (int)g.R, F, out);
            DLC_FSTAMP(11);
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
