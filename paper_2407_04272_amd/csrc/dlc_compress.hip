// Compression kernels for gfx950: quantise + histogram, Huffman codebook, bit-packed encode with
// scanned offsets, finalize.
//
// Mapping used by the streaming kernels: one wavefront owns one group of 64*S symbols; lane l owns
// chunk l of the group and, at turn j, the four symbols  group_base + j*256 + 4*l .. +3  (one 16-byte
// load per lane, 1 KiB contiguous per wavefront instruction).
#include <algorithm>

#include "dlc_codec_dev.h"

namespace dlc {

void launch_encode_64(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch, uint8_t* out,
                      uint64_t capacity, uint32_t bpt, hipStream_t s);
void launch_encode_128(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch, uint8_t* out,
                       uint64_t capacity, uint32_t bpt, hipStream_t s);
void launch_encode_256(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch, uint8_t* out,
                       uint64_t capacity, uint32_t bpt, hipStream_t s);
void launch_encode_carry_64(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch, uint8_t* out,
                            uint64_t capacity, uint32_t bpt, hipStream_t s);
void launch_encode_carry_128(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch, uint8_t* out,
                             uint64_t capacity, uint32_t bpt, hipStream_t s);
void launch_encode_carry_256(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch, uint8_t* out,
                             uint64_t capacity, uint32_t bpt, hipStream_t s);

// ------------------------------------------------------------------------------------------------
// quantiser alone (inspection entry point)
// ------------------------------------------------------------------------------------------------
template <bool F16>
__global__ __launch_bounds__(256) void k_quantize(const void* payload, Geom g, const QParam* qp, uint16_t* sym) {
    const uint32_t t = blockIdx.y;
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < g.n; i += gridDim.x * blockDim.x) {
        float x;
        if constexpr (F16) x = __half2float(__ushort_as_half(reinterpret_cast<const unsigned short*>(tab)[i]));
        else x = reinterpret_cast<const float*>(tab)[i];
        sym[(size_t)t * g.n + i] = (uint16_t)quant_symbol<F16>(x, q, Rf, (int)g.R);
    }
}

hipError_t launch_quantize(const Geom& g, const void* payload, const QParam* qp, uint16_t* sym, hipStream_t s) {
    dim3 grid(std::min<uint32_t>((g.n + 255) / 256, 1024), g.T);
    if (g.dtype == DLC_F16) hipLaunchKernelGGL(k_quantize<true>, grid, dim3(256), 0, s, payload, g, qp, sym);
    else hipLaunchKernelGGL(k_quantize<false>, grid, dim3(256), 0, s, payload, g, qp, sym);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// quantise + histogram
//   grid: T * bpt work-groups of 4 wavefronts; a work-group stays inside one table, counts into its LDS
//   histogram and merges that into the table's global one at the end.
// ------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) uint32_t lds_u32;
__device__ __forceinline__ void lds_count(uint32_t addr) {
    __hip_atomic_fetch_add(reinterpret_cast<lds_u32*>(addr), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

struct HistC {
    int ubias;          // window index of bin 0
    uint32_t win_lo;    // symbol of window index 0
    uint32_t lanebase;  // LDS address of this lane's copy of window row 0
    uint32_t exact;     // LDS address of the exact counts
};

// hook for micro-benchmarks (counting switched off); the library counts

constexpr uint32_t kPastEnd = 0x80000001u;  // no element within the radius has this window index: a position past the end of the table
constexpr uint32_t kHistBlk = 4;  // units whose loads are issued back to back

// One block of kHistBlk units of one table; a unit is 256 consecutive elements (one 16-byte load per lane).
// `rem` = elements of the table from the block's first element on, `n_units` = units of the block that are this
// wavefront's.  FULL: all kHistBlk units are, and all their elements are inside the table (no masking at all).
// Index 254 in the plane stands for an escape.  LZ (row matching): the window is one symbol narrower, because index
// 253 stands for an element of a row that is stored as a reference (the row-matching kernels put it there
// afterwards); the symbol that would have had that index goes the way of everything outside the window.
template <bool F16, bool VEC, bool FULL, bool LZ, bool PLANE = true>
__device__ __forceinline__ void hist_block(const uint8_t* base, uint32_t rem, uint32_t n_units, uint32_t lane, const QParam& q,
                                           float Rf, const HistC& H, uint32_t* plane) {
    constexpr uint32_t kBins = LZ ? kWinSkip : kWinEsc;  // window indices that stand for a symbol
    float x[kHistBlk][4];
    uint32_t raw[kHistBlk][4];
    uint32_t valid[kHistBlk];
#pragma unroll
    for (uint32_t u = 0; u < kHistBlk; ++u) {
        const uint32_t lim = FULL ? 0xFFFFFFFFu : (u < n_units ? rem : 0u);
        valid[u] = load4<F16, VEC>(base, lane * kV + u * (kW * kV), lim, x[u], raw[u]);
    }
#pragma unroll
    for (uint32_t u = 0; u < kHistBlk; ++u) {
        uint32_t w[4], sl[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            // the quantiser (same arithmetic as quant_symbol), result as a window index
            const float xv = x[u][v];
            const float r = __builtin_rintf(xv * q.inv);
            float xh = r * q.ebx2;
            if constexpr (F16) xh = __half2float(half_rne(xh));
            const float d = xv - xh;
            const bool ok = (__builtin_fabsf(r) < Rf) & (__builtin_fabsf(d) <= q.eb);  // no short circuit: no branches
            w[v] = (uint32_t)((int)r + H.ubias);  // (bins below the window wrap to just under 2^32)
            sl[v] = w[v] < kBins ? w[v] : kWinBins;
            sl[v] = ok ? sl[v] : kWinEsc;
            if constexpr (FULL) {
                lds_count(sl[v] * (kWinCopies * 4u) + H.lanebase);
            } else {
                if ((valid[u] >> v) & 1u) lds_count(sl[v] * (kWinCopies * 4u) + H.lanebase);
                else { sl[v] = kWinBins; w[v] = kPastEnd; }
            }
        }
        // index 255 is rare: count those elements exactly, by symbol (escapes are counted in window row 254, which
        // the merge adds to symbol 0)
        if (__ballot(max(max(sl[0], sl[1]), max(sl[2], sl[3])) == kWinBins) != 0ull) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (sl[v] == kWinBins && w[v] != kPastEnd) lds_count(H.exact + (w[v] + H.win_lo) * 4u);
        }
        // the window indices of these four elements, for the encode kernel (a unit of this wavefront only)
        if constexpr (PLANE) {
            if (FULL || u < n_units) plane[u * kW + lane] = sl[0] | (sl[1] << 8) | (sl[2] << 16) | (sl[3] << 24);
        }
    }
}

// The payload is cut into units of 256 elements, U per table, and every wavefront of the grid gets the same
// number of consecutive units (table after table), so that all of them finish together whatever the shape is.
// A work-group whose units touch several tables handles them one table at a time.
// SAMPLE (single-pass path with DLC_FLAG_SAMPLE_CODEBOOK): only a few groups of every table are counted, for the
// codebook; U is then the number of units of a table's sampled groups, unit u of them stands for unit
// (u / upg) * gstride * upg + u % upg of the table (upg = units of a group, gstride = groups from one sampled group
// to the next), and no plane is written.  (Building a table's codebook in the same launch was tried
// both ways: by the work-group that is the last to add its counts, the launch takes as long as the two it replaces;
// by a single work-group per table that also does all the counting, longer.)
struct SampleArgs {
    uint32_t upg, gstride;
};

template <bool F16, bool VEC, bool LZ, bool SAMPLE = false>
__global__ __launch_bounds__(256) void k_hist(const void* payload, Geom g, const QParam* qp, uint32_t* hist,
                                              uint8_t* sym_plane, uint32_t U, uint32_t units_per_wave, SampleArgs sa) {
    extern __shared__ __align__(16) uint32_t lh[];
    const uint32_t upg = sa.upg, gstride = sa.gstride;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lds0 = (uint32_t)(uintptr_t)lh;
    HistC H;
    H.win_lo = win_lo_of(g.R);
    H.ubias = (int)(g.R - H.win_lo);
    H.lanebase = lds0 + (lane & (kWinCopies - 1u)) * 4u;
    H.exact = lds0 + (kWinBins + 1u) * kWinCopies * 4u;
    const uint32_t n_words = (kWinBins + 1u) * kWinCopies + g.K;
    const float Rf = (float)g.R;
    const uint64_t total_units = (uint64_t)g.T * U;
    // this wavefront's units [w0, w1) and the work-group's [g0, g1), as global unit numbers
    const uint64_t g0 = (uint64_t)blockIdx.x * 4u * units_per_wave;
    const uint64_t g1 = min(total_units, g0 + 4ull * units_per_wave);
    const uint64_t w0 = min(total_units, g0 + (uint64_t)wave * units_per_wave), w1 = min(total_units, w0 + units_per_wave);
    if (g0 >= g1) return;  // uniform
    const uint32_t t_first = (uint32_t)(g0 / U), t_last = (uint32_t)((g1 - 1) / U);
    for (uint32_t t = t_first; t <= t_last; ++t) {
        {
            uint4* z = reinterpret_cast<uint4*>(lh);
            for (uint32_t k = tid; k < (n_words + 3u) / 4u; k += 256) z[k] = make_uint4(0, 0, 0, 0);
        }
        __syncthreads();
        const QParam q = qp[t];
        const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
        // my units inside table t
        const uint64_t t0 = (uint64_t)t * U, t1 = t0 + U;
        const uint64_t a = max(w0, t0), b = min(w1, t1);
        if (a < b) {
            uint32_t u = (uint32_t)(a - t0);
            const uint32_t ue = (uint32_t)(b - t0);
            for (; u < ue; u += kHistBlk) {
                uint32_t ur = u;  // (a block of kHistBlk units never straddles two groups: upg is a multiple of it)
                if constexpr (SAMPLE) ur = (u / upg) * gstride * upg + u % upg;
                const uint32_t first = ur * (kW * kV);  // element of the table
                if constexpr (SAMPLE) {
                    if (first >= g.n) continue;  // (the last sampled group may be the table's last, ragged one)
                }
                const uint8_t* base = tab + (size_t)first * g.es;
                const uint32_t rem = g.n - first;
                const uint32_t n_units = min(kHistBlk, ue - u);
                uint32_t* plane = SAMPLE ? nullptr : reinterpret_cast<uint32_t*>(sym_plane + (size_t)t * plane_stride(g) + first);
                if (n_units == kHistBlk && rem >= kHistBlk * kW * kV) hist_block<F16, VEC, true, LZ, !SAMPLE>(base, rem, n_units, lane, q, Rf, H, plane);
                else hist_block<F16, VEC, false, LZ, !SAMPLE>(base, rem, n_units, lane, q, Rf, H, plane);
            }
        }
        __syncthreads();
        // merge: the window rows (sum of the copies, skewed start so that the threads of a wavefront read different
        // banks) plus the exact counts
        const uint32_t* exact = lh + (kWinBins + 1u) * kWinCopies;
        for (uint32_t k = tid; k < g.K; k += 256) {
            uint32_t s = exact[k];
            const uint32_t w = k - H.win_lo;
            if (w < (LZ ? kWinSkip : kWinEsc)) {
                const uint32_t* row = lh + w * kWinCopies;
                for (uint32_t c = 0; c < kWinCopies; ++c) s += row[(c + tid) & (kWinCopies - 1u)];
            }
            if (k == 0u) {  // the escapes
                const uint32_t* row = lh + kWinEsc * kWinCopies;
                for (uint32_t c = 0; c < kWinCopies; ++c) s += row[c];
            }
            if (s) atomicAdd(&hist[(size_t)t * g.K + k], s);
        }
        __syncthreads();
    }
}

// carry != 0: the codebook is for the next call (the escape symbol gets a code whether it occurred or not)
// tpw: tables per work-group, 1 or 4 (see codebook_tables_per_wg)
__global__ __launch_bounds__(256) void k_codebook(Geom g, uint32_t* hist, uint32_t* hist_view, uint16_t* enc,
                                                  uint8_t* lens, TMeta* tmeta, uint32_t carry, uint32_t tpw) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ CodebookShared sh;
    __shared__ uint32_t s_slow[4];
    if (tpw == 4u) {
        codebook_build_four(g, blockIdx.x * 4u, hist, hist_view, enc, lens, tmeta, smem, sh, s_slow, threadIdx.x, carry);
    } else {
        const uint32_t t = blockIdx.x;
        codebook_build(g, hist + (size_t)t * g.K, hist_view + (size_t)t * g.K, enc + (size_t)t * g.K,
                       lens + (size_t)t * g.K, tmeta + t, smem, sh, threadIdx.x, carry);
    }
}

// With few tables a work-group per table (all its threads read the histogram: the shortest way to one codebook); with
// many, four tables per work-group, a wavefront each (a quarter of the work-groups, and no idle wavefronts while
// one of them builds the tree).
static inline uint32_t codebook_tables_per_wg(const Geom& g) { return g.T >= 512u ? 4u : 1u; }

// ------------------------------------------------------------------------------------------------
// finalize: code-length blocks behind the payload, header, directory, padding, size metadata; clears the
// per-call control words for the next call.  Work-groups of 1024 threads: every work-group works out where the
// code-length blocks go (a scan over the tables) and writes the blocks of its share of the tables, a wavefront
// per table; the first work-group also writes everything else.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t a16(uint64_t x) { return (x + 15ull) & ~15ull; }

// One destination's container, by work-group xi of the xn that share the work (all of NT threads); everything below is
// that container's.  The tables' word ranges may come from work-groups of the running kernel: they are read past the caches.
template <uint32_t NT>
__device__ __forceinline__ void finalize_dest(const Geom& g, const FixedLayout& F, const TMeta* tmeta, const uint8_t* __restrict__ lens,
                                              const QParam* qp, Ctrl* ctrl, const uint32_t* word_start, const uint32_t* word_end,
                                              uint8_t* __restrict__ out, uint64_t capacity, uint64_t* out_bytes, uint32_t* esc_count,
                                              const uint8_t* rm_on, const uint32_t* rm_ref, uint32_t* bsum, uint32_t dst, uint32_t xi,
                                              uint32_t xn) {
    constexpr uint32_t NW = NT / 64u;
    __shared__ uint32_t s_red[NW + 1];
    __shared__ uint32_t s_abort;
    __shared__ uint32_t s_cb[NT + 1];   // start of each table's block, relative to the pass's first block
    __shared__ uint32_t s_lo[NT], s_nl[NT];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const bool first = xi == 0;
    const uint32_t T = g.TD;
    tmeta += (size_t)dst * T;
    lens += (size_t)dst * T * g.K;
    qp += (size_t)dst * T;
    word_start += (size_t)dst * T;
    word_end += (size_t)dst * T;
    if (esc_count) esc_count += (size_t)dst * T;
    out += (uint64_t)dst * capacity;
    uint64_t* const table_bytes = out_bytes + 1 + (size_t)dst * T;
    const uint64_t words = __hip_atomic_load(&word_end[T - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint64_t off_cb = a16(F.off_payload + 4ull * words);
    // an internal failure of the encode kernel spoils every container; one that did not fit spoils only itself, and
    // the capacity test below fails for it whenever the encode kernel's did.  (The flag is cleared by the last
    // destination to finish, so every destination's first work-group can still read it.)
    if (first && bsum) {  // single-pass path: the block sums the next call adds to start at zero (not the ones this call reads)
        const uint32_t nb = sum_blocks_per_dest(g);
        for (uint32_t i = tid; i < nb; i += NT) bsum[(size_t)dst * nb + i] = 0u;
    }
    const bool aborted = first && (__hip_atomic_load(&ctrl->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kAbortInternal) != 0;
    uint64_t cb_carry = 0, nout_carry = 0;
    for (uint32_t base = 0; base < T; base += NT) {
        const uint32_t t = base + tid;
        TMeta m;
        uint32_t cb = 0, no = 0, nl = 0;
        if (t < T) {
            m = tmeta[t];
            if (first && esc_count) {  // single-pass path: the codebook is older than the payload, the escapes were counted by the encode kernel
                m.n_outliers = esc_count[t];
                esc_count[t] = 0;
            }
            if (m.sym_lo > m.sym_hi || m.sym_hi >= g.K) { m.sym_lo = 0; m.sym_hi = 0; }  // never index outside lens[]
            nl = m.sym_hi - m.sym_lo + 1u;
            cb = (nl + 3u) & ~3u;
            no = m.n_outliers;
        }
        uint32_t cb_tot, no_tot;
        const uint32_t cb_ex = block_excl_scan<(int)NW>(cb, s_red, tid, &cb_tot);
        __syncthreads();
        (void)block_excl_scan<(int)NW>(no, s_red, tid, &no_tot);
        s_cb[tid] = cb_ex;
        s_lo[tid] = m.sym_lo;
        s_nl[tid] = nl;
        if (tid == 0) {
            s_cb[NT] = cb_tot;
            // the code-length blocks are the last thing in the container: the capacity check of this pass
            s_abort = aborted || off_cb + cb_carry + cb_tot > capacity;
        }
        __syncthreads();
        if (s_abort) break;  // uniform
        const uint32_t nt = min(NT, T - base);
        // the blocks of this work-group's tables, a wavefront per table, four bytes per lane (the blocks start on
        // 4-byte boundaries and are padded to them)
        for (uint32_t lt = xi * NW + wave; lt < nt; lt += xn * NW) {
            const uint32_t n_l = s_nl[lt];
            const uint8_t* src = lens + (size_t)(base + lt) * g.K + s_lo[lt];
            uint32_t* dst = reinterpret_cast<uint32_t*>(out + off_cb + cb_carry + s_cb[lt]);
            for (uint32_t wd = lane; wd < (n_l + 3u) / 4u; wd += 64) {
                uint32_t v = 0;
#pragma unroll
                for (uint32_t b = 0; b < 4; ++b) {
                    const uint32_t i = wd * 4u + b;
                    v |= (i < n_l ? (uint32_t)src[i] : 0u) << (8u * b);
                }
                dst[wd] = v;
            }
        }
        if (first && t < T) {
            const uint64_t w0 = __hip_atomic_load(&word_start[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint64_t w1 = __hip_atomic_load(&word_end[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            uint8_t* d = out + kHeaderBytes + (uint64_t)kDirBytes * t;
            uint32_t* d32 = reinterpret_cast<uint32_t*>(d);
            d32[0] = qp[t].eb_bits; d32[1] = m.n_used; d32[2] = m.sym_lo; d32[3] = m.sym_hi; d32[4] = m.n_outliers;
            d32[5] = g.G;
            uint64_t* d64 = reinterpret_cast<uint64_t*>(d + 24);
            d64[0] = off_cb + cb_carry + cb_ex; d64[1] = 0; d64[2] = w0; d64[3] = w1 - w0;
            table_bytes[t] = 4ull * (w1 - w0) + cb + (uint64_t)(kW + 4u) * g.G + kDirBytes;
        }
        cb_carry += cb_tot;
        nout_carry += no_tot;
        __syncthreads();
    }
    // row matching: the references of the tables that use it, behind the code-length blocks, each block on a 16-byte
    // boundary (all blocks are 4*B bytes, so block k starts k * a16(4*B) after the first)
    uint64_t end_bytes = off_cb + cb_carry;  // where the container ends
    if (rm_on && !s_abort) {
        rm_on += (size_t)dst * T;
        rm_ref += (size_t)dst * T * g.B;
        const uint64_t rbase = a16(end_bytes), rsz = a16(4ull * g.B);
        uint32_t n_on = 0;  // tables with references
        for (uint32_t base = 0; base < T; base += NT) {
            uint32_t tot;
            (void)block_excl_scan<(int)NW>((base + tid < T && rm_on[base + tid]) ? 1u : 0u, s_red, tid, &tot);
            n_on += tot;
            __syncthreads();
        }
        if (n_on) end_bytes = rbase + (uint64_t)(n_on - 1u) * rsz + 4ull * g.B;
        if (end_bytes > capacity) {  // uniform
            __syncthreads();
            if (tid == 0) s_abort = 1;
            __syncthreads();
        } else if (n_on) {
            for (uint64_t i = off_cb + cb_carry + tid; first && i < rbase; i += NT) out[i] = 0;
            uint32_t on_carry = 0;
            for (uint32_t base = 0; base < T; base += NT) {
                const uint32_t t = base + tid;
                const uint32_t on = (t < T && rm_on[t]) ? 1u : 0u;
                uint32_t tot;
                const uint32_t ex = block_excl_scan<(int)NW>(on, s_red, tid, &tot);
                s_cb[tid] = on ? on_carry + ex : 0xFFFFFFFFu;  // the table's block number
                __syncthreads();
                if (first && on) {
                    uint64_t* d64 = reinterpret_cast<uint64_t*>(out + kHeaderBytes + (uint64_t)kDirBytes * t + 24);
                    d64[1] = rbase + (uint64_t)(on_carry + ex) * rsz;
                    table_bytes[t] += 4ull * g.B;
                }
                const uint32_t nt = min(NT, T - base);
                for (uint32_t lt = xi; lt < nt; lt += xn) {  // a work-group per table
                    const uint32_t k = s_cb[lt];
                    if (k == 0xFFFFFFFFu) continue;  // uniform
                    uint32_t* dstw = reinterpret_cast<uint32_t*>(out + rbase + (uint64_t)k * rsz);
                    const uint32_t* src = rm_ref + (size_t)(base + lt) * g.B;
                    for (uint32_t r = tid; r < g.B; r += NT) dstw[r] = src[r];
                    if (k + 1u < n_on)  // padding up to the next block
                        for (uint32_t r = g.B + tid; r < (uint32_t)(rsz / 4u); r += NT) dstw[r] = 0u;
                }
                on_carry += tot;
                __syncthreads();
            }
        }
    }
    if (!first) return;
    uint64_t container_bytes = 0;  // of this destination; 0 = it did not fit
    if (s_abort) {
        if (tid == 0 && !aborted) set_status(ctrl, DLC_ECAPACITY);
        for (uint32_t t = tid; t < T; t += NT) table_bytes[t] = 0;
        if (esc_count)  // whatever the passes after the failing one have not cleared
            for (uint32_t t = tid; t < T; t += NT) esc_count[t] = 0;
    } else {
        // padding between sections
        const uint64_t e0 = kHeaderBytes + (uint64_t)kDirBytes * T;
        for (uint64_t i = e0 + tid; i < F.off_group; i += NT) out[i] = 0;
        const uint64_t e1 = F.off_group + 4ull * T * g.G;
        for (uint64_t i = e1 + tid; i < F.off_chunk; i += NT) out[i] = 0;
        const uint64_t e2 = F.off_payload + 4ull * words;
        for (uint64_t i = e2 + tid; i < off_cb; i += NT) out[i] = 0;
        if (tid == 0) {
            uint32_t* h = reinterpret_cast<uint32_t*>(out);
            h[H_MAGIC] = kMagic; h[H_VERSION] = kVersion; h[H_DTYPE] = g.dtype; h[H_T] = T; h[H_B] = g.B; h[H_D] = g.D;
            h[H_R] = g.R; h[H_S] = g.S; h[H_LMAX] = g.LMAX; h[H_W] = kW; h[H_V] = kV; h[H_NG] = T * g.G;
            uint64_t* q = reinterpret_cast<uint64_t*>(out);
            q[HQ_NOUT] = nout_carry; q[HQ_WORDS] = words; q[HQ_OFF_GROUP] = F.off_group; q[HQ_OFF_CHUNK] = F.off_chunk;
            q[HQ_OFF_PAYLOAD] = F.off_payload; q[HQ_OFF_CB] = off_cb;
            const uint64_t total = end_bytes;
            q[HQ_TOTAL] = total; q[HQ_TOTAL + 1] = 0; q[HQ_TOTAL + 2] = 0; q[HQ_TOTAL + 3] = 0;
            container_bytes = total;
        }
    }
    if (tid != 0) return;
    // sizes: one destination -> out_bytes[0] is its container's size.  Several -> every destination stores its size
    // behind the per-table entries, and the last one to do so adds them up into out_bytes[0] (0 if any did not fit).
    // the next call starts with ticket 0 and no abort (the histograms were cleared by the codebook step)
    if (g.ND == 1) {
        out_bytes[0] = container_bytes;
        ctrl->ticket = 0;
        ctrl->abort = 0;
    } else {
        unsigned long long* dest_bytes = reinterpret_cast<unsigned long long*>(out_bytes + 1 + (size_t)g.ND * T);
        __hip_atomic_store(&dest_bytes[dst], (unsigned long long)container_bytes, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (__hip_atomic_fetch_add(&ctrl->dest_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == g.ND) {
            unsigned long long sum = 0;
            bool all = true;
            for (uint32_t d = 0; d < g.ND; ++d) {
                const unsigned long long b = __hip_atomic_load(&dest_bytes[d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                all = all && b != 0;
                sum += b;
            }
            out_bytes[0] = all ? sum : 0;
            __hip_atomic_store(&ctrl->dest_done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ctrl->ticket = 0;
            __hip_atomic_store(&ctrl->abort, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

__global__ __launch_bounds__(1024) void k_finalize(Geom g, FixedLayout F, const TMeta* tmeta, const uint8_t* __restrict__ lens,
                                                   const QParam* qp, Ctrl* ctrl, const uint32_t* word_start,
                                                   const uint32_t* word_end, uint8_t* __restrict__ out, uint64_t capacity,
                                                   uint64_t* out_bytes, uint32_t* esc_count, const uint8_t* rm_on,
                                                   const uint32_t* rm_ref, uint32_t* bsum) {
    // blockIdx.y: the destination whose container this work-group helps to finish
    finalize_dest<1024>(g, F, tmeta, lens, qp, ctrl, word_start, word_end, out, capacity, out_bytes, esc_count, rm_on, rm_ref, bsum,
                        blockIdx.y, blockIdx.x, gridDim.x);
}

// ------------------------------------------------------------------------------------------------
// single-pass path, second step: one launch, three jobs that do not wait for one another.  Where a group's words go
// is the sum of the totals of all groups before it in its container; the encode kernel has added the totals up per
// block of kSumBlock groups, so whoever needs such a sum reads the sums of the blocks before and the totals of the
// groups in between.
//   the first work-groups, one per table or per four tables: the codebook of the next call from this call's counts, into the second set of codebook arrays
//     (this call's set is still being read)
//   then nf work-groups per destination: the container's header, directory, code-length blocks, sizes (finalize_dest),
//     from the tables' word ranges, which they work out from the sums themselves
//   the rest: the groups' words from their slots to their places, kPlaceGroups groups per work-group, a group per
//     wavefront (coalesced both ways), and the group table.  Nothing is written past a container's capacity.
// ------------------------------------------------------------------------------------------------
// words of the groups [0, x) of a destination (called by a whole wavefront, same x)
__device__ __forceinline__ unsigned long long words_before(const uint32_t* bs, const uint32_t* gtot_d, uint32_t x, uint32_t lane) {
    const uint32_t blk = x / kSumBlock;
    unsigned long long acc = 0;
    for (uint32_t i = lane; i < blk; i += 64) acc += bs[i];
    for (uint32_t i = blk * kSumBlock + lane; i < x; i += 64) acc += gtot_d[i];
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    return acc;
}

__global__ __launch_bounds__(256) void k_post(Geom g, FixedLayout F, const uint32_t* gtot, const uint32_t* bsum, uint32_t* bsum_next,
                                              const uint32_t* slots, uint64_t slot_words, Ctrl* ctrl, uint8_t* out,
                                              uint64_t capacity, uint32_t wpd, uint32_t nf, uint32_t* word_start,
                                              uint32_t* word_end, const TMeta* tmeta, const uint8_t* lens, const QParam* qp,
                                              uint64_t* out_bytes, uint32_t* esc_count, uint32_t* hist, uint32_t* hist_view,
                                              uint16_t* enc_next, uint8_t* lens_next, TMeta* tmeta_next, uint32_t tpw) {
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t gpd = g.TD * g.G;  // groups of one destination
    // work-groups that build the next call's codebooks, tpw (1 or 4) tables each; tpw == 0: none (no codebook is carried)
    const uint32_t n_cb = tpw ? (g.T + tpw - 1u) / tpw : 0u;
    if (blockIdx.x < n_cb) {  // uniform over the work-group; these come first: a codebook takes longer than a copy
        __shared__ CodebookShared sh;
        __shared__ uint32_t s_slow[4];
        if (tpw == 4u) {
            codebook_build_four(g, blockIdx.x * 4u, hist, hist_view, enc_next, lens_next, tmeta_next, smem, sh, s_slow, tid, 1u);
        } else {
            const uint32_t t = blockIdx.x;
            codebook_build(g, hist + (size_t)t * g.K, hist_view + (size_t)t * g.K, enc_next + (size_t)t * g.K,
                           lens_next + (size_t)t * g.K, tmeta_next + t, smem, sh, tid, 1u);
        }
        return;
    }
    if (blockIdx.x < n_cb + g.ND * nf) {
        const uint32_t f = blockIdx.x - n_cb, dst = f / nf, xi = f - dst * nf;
        const uint32_t* const bs = bsum + (size_t)dst * sum_blocks_per_dest(g);
        const uint32_t* const gtot_d = gtot + (size_t)dst * gpd;
        // The tables' word ranges (stored past the caches: finalize_dest reads them that way): a scan over the block
        // sums, 256 blocks a pass; the thread of a block looks after the tables that start inside it.  Every one of
        // the nf work-groups needs the last table's end, only the first of them the rest.
        __shared__ uint32_t s_scan[5];
        __shared__ unsigned long long s_sum64[4];
        const uint32_t nb = sum_blocks_per_dest(g);
        uint32_t carry = 0;
        unsigned long long all = 0;
        for (uint32_t c0 = 0; c0 < nb; c0 += 256) {  // uniform trip count
            const uint32_t blk = c0 + tid;
            const uint32_t v = blk < nb ? bs[blk] : 0u;
            unsigned long long v64 = v;
            for (int o = 32; o > 0; o >>= 1) v64 += __shfl_xor(v64, o, 64);
            if (lane == 0) s_sum64[wave] = v64;
            uint32_t tot;
            const uint32_t before = carry + block_excl_scan<4>(v, s_scan, tid, &tot);
            all += s_sum64[0] + s_sum64[1] + s_sum64[2] + s_sum64[3];
            if (xi == 0 && blk < nb) {
                const uint32_t x0 = blk * kSumBlock, x1 = min(gpd, x0 + kSumBlock);
                uint32_t w = before, i = x0;  // (one walk over the block's groups serves all the tables that start in it)
                for (uint32_t tl = (x0 + g.G - 1u) / g.G; tl < g.TD && tl * g.G < x1; ++tl) {
                    for (; i < tl * g.G; ++i) w += gtot_d[i];
                    __hip_atomic_store(&word_start[dst * g.TD + tl], w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (tl > 0) __hip_atomic_store(&word_end[dst * g.TD + tl - 1u], w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            carry += tot;
            __syncthreads();
        }
        if (tid == 0) {  // (clamped; past 2^32 words the format cannot say where a group starts: the call fails)
            if (all > 0xFFFFFFFFull && xi == 0) { set_status(ctrl, DLC_ECAPACITY); atomicOr(&ctrl->abort, kAbortInternal); }
            __hip_atomic_store(&word_end[dst * g.TD + g.TD - 1u], (uint32_t)min(all, 0xFFFFFFFFull), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        finalize_dest<256>(g, F, tmeta, lens, qp, ctrl, word_start, word_end, out, capacity, out_bytes, esc_count,
                           (const uint8_t*)nullptr, (const uint32_t*)nullptr, bsum_next, dst, xi, nf);
        return;
    }
    const uint32_t wg = blockIdx.x - n_cb - g.ND * nf;
    const uint32_t dst = wg / wpd, k = wg - dst * wpd;  // wpd work-groups per destination
    const uint32_t g0 = k * kPlaceGroups;
    if (g0 + wave >= gpd) return;  // whole wavefront
    uint8_t* const out_d = out + (uint64_t)dst * capacity;
    const uint32_t gl = g0 + wave;  // group number inside the container
    const size_t gg = (size_t)dst * gpd + gl;
    const unsigned long long base = words_before(bsum + (size_t)dst * sum_blocks_per_dest(g), gtot + (size_t)dst * gpd, gl, lane);
    const uint32_t total = gtot[gg];
    // (word offsets are 32-bit: a container of 2^32 words or more does not fit any capacity the format can describe;
    // the finishing work-groups come to the same verdict from the same sums and report it)
    if (base + total > 0xFFFFFFFFull || F.off_payload + 4ull * (base + total) > capacity) return;  // uniform over the wavefront
    const uint32_t goff = (uint32_t)base;
    if (lane == 0) reinterpret_cast<uint32_t*>(out_d + F.off_group)[gl] = goff;
    const uint32_t* src = slots + gg * slot_words;
    uint32_t* dstw = reinterpret_cast<uint32_t*>(out_d + F.off_payload) + goff;
    uint32_t j = lane;
    for (; j + 448u < total; j += 512u) {  // eight loads in flight
        uint32_t v[8];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) v[u] = src[j + 64u * u];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) dstw[j + 64u * u] = v[u];
    }
    {  // the rest: up to eight more, all in flight too
        uint32_t v[8];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) v[u] = j + 64u * u < total ? src[j + 64u * u] : 0u;
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u)
            if (j + 64u * u < total) dstw[j + 64u * u] = v[u];
    }
}

// work-groups of the finalize kernel: a wavefront per table, sixteen wavefronts per work-group
static inline dim3 finalize_grid(const Geom& g) {
    // a wavefront per table for the code-length blocks; with row matching a work-group per table copies its references
    const uint32_t per_wg = g.lz ? 1u : 16u;
    return dim3(std::min<uint32_t>((std::min<uint32_t>(g.TD, 1024u) + per_wg - 1u) / per_wg, 64u), g.ND);
}

hipError_t launch_compress(const Geom& g, const void* payload, uint8_t* out, uint64_t capacity, uint64_t* out_bytes,
                           const Ws& w, uint64_t epoch, bool carry_ready, int pl, void* prof, hipStream_t s) {
    const bool f16 = g.dtype == DLC_F16;
    const FixedLayout F = fixed_layout(g);
    if (w.sample != 0) {
        // single pass without a carried codebook: the counts of a few groups of every table, their codebook (the escape
        // symbol always gets a code: an element whose symbol the sample has not seen is stored as an escape)
        uint32_t ns, gstride;
        sample_groups(g, &ns, &gstride);
        const uint32_t upg = g.S / kV;  // units of a group
        const uint32_t U = ns * upg;
        const uint64_t total_units = (uint64_t)g.T * U;
        const uint32_t units_per_wave = 4 * kHistBlk;
        const uint32_t grid_n = (uint32_t)((total_units + 4ull * units_per_wave - 1) / (4ull * units_per_wave));
        SampleArgs sa;
        sa.upg = upg; sa.gstride = gstride;
        const size_t sm = hist_lds_bytes(g.K);
        if (prof_on(pl, P_HIST)) prof_begin(prof, P_HIST, s);
#define DLC_HIST(FF, V) hipLaunchKernelGGL((k_hist<FF, V, false, true>), dim3(grid_n), dim3(256), sm, s, payload, g, w.qp, w.hist, \
                                           (uint8_t*)nullptr, U, units_per_wave, sa)
        if (f16) { if (g.vec) DLC_HIST(true, true); else DLC_HIST(true, false); }
        else { if (g.vec) DLC_HIST(false, true); else DLC_HIST(false, false); }
#undef DLC_HIST
        if (prof_on(pl, P_HIST)) prof_end(prof, P_HIST, s);
        if (prof_on(pl, P_CODEBOOK)) prof_begin(prof, P_CODEBOOK, s);
        const uint32_t tpw = codebook_tables_per_wg(g);
        hipLaunchKernelGGL(k_codebook, dim3((g.T + tpw - 1u) / tpw), dim3(256), codebook_smem(g.K), s, g, w.hist, w.hist_view, w.enc, w.lens,
                           w.tmeta, 1u, tpw);
        if (prof_on(pl, P_CODEBOOK)) prof_end(prof, P_CODEBOOK, s);
    }
    if (w.sample != 0 || (w.carry != 0 && carry_ready)) {
        // single pass: encode with the codebook of the previous call, then build the next one from this call's counts
        // (or, with the sample's codebook, nothing to build)
        const uint32_t bpt = (g.G + 3) / 4;
        if (prof_on(pl, P_CARRY)) prof_begin(prof, P_CARRY, s);
        switch (g.S) {
            case 64: launch_encode_carry_64(g, F, payload, w, epoch, out, capacity, bpt, s); break;
            case 128: launch_encode_carry_128(g, F, payload, w, epoch, out, capacity, bpt, s); break;
            default: launch_encode_carry_256(g, F, payload, w, epoch, out, capacity, bpt, s); break;
        }
        if (prof_on(pl, P_CARRY)) prof_end(prof, P_CARRY, s);
        {
            const uint32_t wpd = (g.TD * g.G + kPlaceGroups - 1) / kPlaceGroups, n_place = g.ND * wpd;
            const uint32_t nf = std::min<uint32_t>((std::min<uint32_t>(g.TD, 256u) + 3u) / 4u, 64u);  // a wavefront per table's code-length block
            if (prof_on(pl, P_POST)) prof_begin(prof, P_POST, s);
            const uint32_t tpw = w.sample != 0 ? 0u : codebook_tables_per_wg(g);
            hipLaunchKernelGGL(k_post, dim3((tpw ? (g.T + tpw - 1u) / tpw : 0u) + g.ND * nf + n_place), dim3(256), codebook_smem(g.K), s, g, F, w.gtot, w.bsum,
                               w.bsum_next, w.slots, (uint64_t)carry_slot_words(g), w.ctrl, out, capacity, wpd, nf, w.word_start,
                               w.word_end, w.tmeta, w.lens, w.qp, out_bytes, w.esc_count, w.hist, w.hist_view, w.enc_next,
                               w.lens_next, w.tmeta_next, tpw);
            if (prof_on(pl, P_POST)) prof_end(prof, P_POST, s);
        }
        return hipGetLastError();
    }
    // histogram
    {
        // equal shares of 16 units (16 KiB of fp32) per wavefront: measured best on MI355X, a little ahead of one
        // share per resident wavefront
        const uint32_t U = (g.n + kW * kV - 1) / (kW * kV);
        const uint64_t total_units = (uint64_t)g.T * U;
        const uint32_t units_per_wave = 4 * kHistBlk;
        const uint32_t grid_n = (uint32_t)((total_units + 4ull * units_per_wave - 1) / (4ull * units_per_wave));
        const size_t sm = hist_lds_bytes(g.K);
        dim3 grid(grid_n), block(256);
        if (prof_on(pl, P_HIST)) prof_begin(prof, P_HIST, s);
#define DLC_HIST(FF, V, L) hipLaunchKernelGGL((k_hist<FF, V, L>), grid, block, sm, s, payload, g, w.qp, w.hist, w.sym_plane, U, units_per_wave, SampleArgs{})
        if (g.lz) {  // row matching wants D % 4 == 0, which makes every table start 16-byte aligned with n % 4 == 0
            if (f16) DLC_HIST(true, true, true); else DLC_HIST(false, true, true);
        } else if (f16) { if (g.vec) DLC_HIST(true, true, false); else DLC_HIST(true, false, false); }
        else { if (g.vec) DLC_HIST(false, true, false); else DLC_HIST(false, false, false); }
#undef DLC_HIST
        if (prof_on(pl, P_HIST)) prof_end(prof, P_HIST, s);
    }
    if (g.lz) {  // row matching: which rows repeat an earlier one; their elements leave the plane and the counts again
        hipError_t e = launch_row_match(g, payload, w, s);
        if (e != hipSuccess) return e;
    }
    if (prof_on(pl, P_CODEBOOK)) prof_begin(prof, P_CODEBOOK, s);
    const uint32_t tpw = codebook_tables_per_wg(g);
    hipLaunchKernelGGL(k_codebook, dim3((g.T + tpw - 1u) / tpw), dim3(256), codebook_smem(g.K), s, g, w.hist, w.hist_view, w.enc, w.lens,
                       w.tmeta, 0u, tpw);
    if (prof_on(pl, P_CODEBOOK)) prof_end(prof, P_CODEBOOK, s);
    {
        const uint32_t bpt = (g.G + 3) / 4;
        if (prof_on(pl, P_ENCODE)) prof_begin(prof, P_ENCODE, s);
        switch (g.S) {
            case 64: launch_encode_64(g, F, payload, w, epoch, out, capacity, bpt, s); break;
            case 128: launch_encode_128(g, F, payload, w, epoch, out, capacity, bpt, s); break;
            default: launch_encode_256(g, F, payload, w, epoch, out, capacity, bpt, s); break;
        }
        if (prof_on(pl, P_ENCODE)) prof_end(prof, P_ENCODE, s);
    }
    if (prof_on(pl, P_FINALIZE)) prof_begin(prof, P_FINALIZE, s);
    hipLaunchKernelGGL(k_finalize, finalize_grid(g), dim3(1024), 0, s, g, F, w.tmeta, w.lens, w.qp, w.ctrl, w.word_start,
                       w.word_end, out, capacity, out_bytes, (uint32_t*)nullptr, g.lz ? (const uint8_t*)w.rm_on : nullptr, (const uint32_t*)w.rm_ref, (uint32_t*)nullptr);
    if (prof_on(pl, P_FINALIZE)) prof_end(prof, P_FINALIZE, s);
    if (w.carry != 0)  // the codebook the next call will use: this call's counts (kept as the copy), escape symbol included
        hipLaunchKernelGGL(k_codebook, dim3((g.T + tpw - 1u) / tpw), dim3(256), codebook_smem(g.K), s, g, w.hist_view, w.hist_view, w.enc_next,
                           w.lens_next, w.tmeta_next, 1u, tpw);
    return hipGetLastError();
}

hipError_t compress_set_attributes() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_codebook), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)codebook_smem(4096));
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_post), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)codebook_smem(4096));
    return e;
}

}  // namespace dlc
