// The encode kernel for one chunk size S (DLC_S, defined by the including source file: one file per S keeps
// the compile times apart).
#include "dlc_codec_dev.h"

#define DLC_CAT2(a, b) a##b
#define DLC_CAT(a, b) DLC_CAT2(a, b)

// phase time stamps of one work-group, for micro-benchmarks only (compiled out of the library)
#ifdef DLC_EXP_STAMPS
__device__ long long g_estamp[32];
#define DLC_ESTAMP(i) do { if (wg == DLC_EXP_STAMPS && threadIdx.x == 0) g_estamp[i] = wall_clock64(); } while (0)
extern "C" void dlc_debug_stamps(long long* out) { (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_estamp), sizeof(g_estamp)); }
#else
#define DLC_ESTAMP(i)
#endif

namespace dlc {

// ------------------------------------------------------------------------------------------------
// bit-packed encode.
//   walk 1: load, quantise, look the (length, codeword) pairs up in LDS, keep them packed in registers,
//           sum the chunk's bits, count the escapes
//   scan  : chunk word counts inside the wavefront; the wavefronts' totals (chunk words + two words per
//           escape) are joined per work-group, and the work-groups' totals across the grid by a single-pass
//           look-back (ordered work-group ids: a work-group only ever waits for work-groups that started
//           earlier)
//   walk 2: shift the kept pairs into a 64-bit accumulator, store whole words at the chunk's offset
//   escapes (rare for fp32): a group that has any walks its elements once more in a rolled loop and
//           writes its records, in increasing element index, behind its chunk words
// ------------------------------------------------------------------------------------------------
template <int S, bool F16, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(S == 256 ? 2 : (S == 128 ? 3 : 5))))
void k_encode(const void* payload, Geom g, FixedLayout F, const QParam* qp, const uint16_t* enc, Ctrl* ctrl,
              uint64_t* state, uint64_t epoch, uint8_t* out, uint64_t capacity, uint32_t bpt, uint32_t* word_start,
              uint32_t* word_end) {
    extern __shared__ __align__(16) uint16_t s_enc[];
    __shared__ uint32_t s_wg, s_tot[4], s_excl, s_dead;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid == 0) s_wg = atomicAdd(&ctrl->ticket, 1u);
    __syncthreads();
    const uint32_t wg = __builtin_amdgcn_readfirstlane(s_wg);
    const uint32_t t = wg / bpt, b = wg % bpt;
    DLC_ESTAMP(0);
    for (uint32_t k = tid; k < g.K; k += 256) s_enc[k] = enc[(size_t)t * g.K + k];
    __syncthreads();
    const uint32_t grp = b * 4 + wave;
    const bool active = grp < g.G;  // uniform over the wavefront; an idle wavefront only takes part in the barriers
    const uint32_t gid = t * g.G + (active ? grp : 0u);
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t gstart = grp * (kW * (uint32_t)S);
    const uint8_t* gbase = tab + (size_t)gstart * g.es;
    const uint32_t rem = active ? g.n - gstart : 0u;

    DLC_ESTAMP(1);
    uint32_t pk[S / 2];
    uint32_t bits = 0;
    uint32_t n_esc = 0;  // escapes of the whole group (a scalar: counted from the comparison masks)
    constexpr int kBlk = 8;  // turns per block (8 x 16 B per lane); the next block's loads are issued before this one is used
    constexpr int kNBlk = S / 4 / kBlk;
    if (active) {
        float x[2][kBlk][4];
        uint32_t raw[2][kBlk][4];
        uint32_t valid[2][kBlk];
#pragma clang loop unroll(full)
        for (int u = 0; u < kBlk; ++u)
            valid[0][u] = load4<F16, VEC>(gbase, lane * kV + (uint32_t)u * (kW * kV), rem, x[0][u], raw[0][u]);
#pragma clang loop unroll(full)
        for (int ib = 0; ib < kNBlk; ++ib) {
            const int cur = ib & 1, nxt = cur ^ 1;
            if (ib + 1 < kNBlk) {
#pragma clang loop unroll(full)
                for (int u = 0; u < kBlk; ++u)
                    valid[nxt][u] = load4<F16, VEC>(gbase, lane * kV + (uint32_t)((ib + 1) * kBlk + u) * (kW * kV), rem, x[nxt][u],
                                                    raw[nxt][u]);
            }
            __builtin_amdgcn_sched_barrier(0);  // the loads above stay above, the work below stays below
#pragma clang loop unroll(full)
            for (int u = 0; u < kBlk; ++u) {
                uint32_t e[4];
#pragma clang loop unroll(full)
                for (int v = 0; v < 4; ++v) {
                    const uint32_t c = quant_symbol<F16>(x[cur][u][v], q, Rf, (int)g.R);
                    const bool ok = (valid[cur][u] >> v) & 1u;
                    // unconditional table read, masked afterwards: a position past the end contributes no bits
                    e[v] = (uint32_t)s_enc[c] & (0u - (uint32_t)ok);
                    n_esc += (uint32_t)__popcll(__ballot(ok && c == 0u));
                }
                uint32_t w0 = e[0] | (e[1] << 16), w1 = e[2] | (e[3] << 16);
                // opaque to the optimiser: otherwise it keeps length and codeword of every symbol in registers of
                // their own instead of the packed words
                asm volatile("" : "+v"(w0), "+v"(w1));
                pk[2 * (ib * kBlk + u)] = w0;
                pk[2 * (ib * kBlk + u) + 1] = w1;
                bits += ((w0 >> 12) & 0xFu) + (w0 >> 28) + ((w1 >> 12) & 0xFu) + (w1 >> 28);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    DLC_ESTAMP(2);
    const uint32_t nw = (bits + 31u) >> 5;
    const uint32_t incl = wave_incl_scan(nw, lane);
    const uint32_t lane_off = incl - nw;
    const uint32_t chunk_total = __shfl(incl, 63, 64);
    const uint32_t total = chunk_total + 2u * n_esc;  // 0 for an idle wavefront

    // offsets: one scan record per work-group; the wavefronts' totals are joined through LDS
    bool dead = false;  // nothing may be written to the container
    if (lane == 0) s_tot[wave] = total;
    __syncthreads();
    if (wave == 0) {
        const uint32_t e = wg_scan(state, epoch, wg, s_tot[0] + s_tot[1] + s_tot[2] + s_tot[3], lane, ctrl, &dead);
        if (lane == 0) { s_excl = e; s_dead = dead ? 1u : 0u; }
    }
    __syncthreads();
    if (!active) return;
    dead = s_dead != 0u;
    uint32_t excl = s_excl;
    for (uint32_t k = 0; k < wave; ++k) excl += s_tot[k];
    DLC_ESTAMP(3);
    if (F.off_payload + 4ull * ((uint64_t)excl + total) > capacity) {
        if (!dead && lane == 0) { set_status(ctrl, DLC_ECAPACITY); ctrl->abort = 1; }
        dead = true;
    }
    if (lane == 0) {
        if (grp == 0) word_start[t] = excl;
        if (grp == g.G - 1) word_end[t] = excl + total;
    }
    if (dead) return;
    emit_group<S, F16, VEC>(pk, nw, lane_off, excl, chunk_total, n_esc, gid, lane, gbase, gstart, rem, q, Rf, (int)g.R, F,
                            out);
    DLC_ESTAMP(4);
}

void DLC_CAT(launch_encode_, DLC_S)(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch,
                                    uint8_t* out, uint64_t capacity, uint32_t bpt, hipStream_t s) {
    constexpr int S = DLC_S;
    dim3 grid(g.T * bpt), block(256);
    const size_t sm = (size_t)g.K * 2;
    const bool f16 = g.dtype == DLC_F16;
#define DLC_ENC(FF, V)                                                                                          \
    hipLaunchKernelGGL((k_encode<S, FF, V>), grid, block, sm, s, payload, g, F, w.qp, w.enc, w.ctrl, w.state, epoch, \
                       out, capacity, bpt, w.word_start, w.word_end)
    if (f16) { if (g.vec) DLC_ENC(true, true); else DLC_ENC(true, false); }
    else { if (g.vec) DLC_ENC(false, true); else DLC_ENC(false, false); }
#undef DLC_ENC
}

}  // namespace dlc
