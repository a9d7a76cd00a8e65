// Compression kernels for gfx950: quantise + histogram, Huffman codebook, bit-packed encode with
// scanned offsets, finalize.
//
// Mapping used by the streaming kernels: one wavefront owns one group of 64*S symbols; lane l owns
// chunk l of the group and, at turn j, the four symbols  group_base + j*256 + 4*l .. +3  (one 16-byte
// load per lane, 1 KiB contiguous per wavefront instruction).
#include <algorithm>

#include "dlc_internal.h"

// phase time stamps for kernel micro-benchmarks; expands to nothing in the library
#ifndef DLC_STAMP
#define DLC_STAMP(i)
#endif

namespace dlc {

// ------------------------------------------------------------------------------------------------
// clear the per-call part of the workspace
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_zero(uint4* p, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

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
// quantise + LDS-privatised histogram
//   grid: T * bpt work-groups of 4 wavefronts; a work-group stays inside one table
//   LDS : LDS atomics with 64 scattered addresses cost one pass per lane that shares a bank, and that -- not
//         HBM, not the ALU -- bounds this kernel.  So the bins around the centre of the alphabet (where a
//         bell-shaped distribution puts almost everything) get 32 copies each, copy = lane & 31: the bank of
//         an update is then the lane's own, whatever its symbol, and a wavefront's 64 updates take the minimum
//         of two passes.  Symbols outside that window go to a single-copy array (rare), positions past the end
//         of the table to a scratch word per lane.
//         layout in words: window [kHistWin][32] | overflow [K] | scratch [64]
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kHistBlk = 4;    // turns whose loads are issued back to back (S/4 is a multiple)
constexpr uint32_t kHistWin = 256;  // bins with private copies (all of them when K <= 256)
constexpr uint32_t kHistCopies = 32;

struct HistLds {
    uint32_t win_bins, win_lo;   // window = symbols [win_lo, win_lo + win_bins)
    uint32_t ovf_byte, trash_byte;  // byte offsets of the overflow array and of this lane's scratch word
};

// FULL: every position of the group is inside the table (no masking at all)
template <bool F16, bool VEC, bool FULL>
__device__ __forceinline__ void hist_group(const uint8_t* gbase, uint32_t rem, uint32_t turns, uint32_t lane,
                                           const QParam& q, float Rf, int R, uint32_t* lh, const HistLds& H) {
    const uint32_t copy4 = (lane & (kHistCopies - 1u)) * 4u;
    for (uint32_t jb = 0; jb < turns; jb += kHistBlk) {
        float x[kHistBlk][4];
        uint32_t raw[kHistBlk][4];
        uint32_t valid[kHistBlk];
#pragma unroll
        for (uint32_t u = 0; u < kHistBlk; ++u)
            valid[u] = load4<F16, VEC>(gbase, lane * kV + (jb + u) * (kW * kV), FULL ? 0xFFFFFFFFu : rem, x[u], raw[u]);
#pragma unroll
        for (uint32_t u = 0; u < kHistBlk; ++u) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const uint32_t c = quant_symbol<F16>(x[u][v], q, Rf, R);
                const uint32_t w = c - H.win_lo;  // wraps for symbols below the window
                uint32_t byte = w < H.win_bins ? w * (kHistCopies * 4u) + copy4 : H.ovf_byte + c * 4u;
                if constexpr (!FULL) byte = ((valid[u] >> v) & 1u) ? byte : H.trash_byte;
                atomicAdd(reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(lh) + byte), 1u);
            }
        }
    }
}

__host__ __device__ inline uint32_t hist_win_bins(uint32_t K) { return K < kHistWin ? K : kHistWin; }
__host__ __device__ inline size_t hist_lds_bytes(uint32_t K) { return ((size_t)hist_win_bins(K) * kHistCopies + K + kW) * 4; }

template <bool F16, bool VEC>
__global__ __launch_bounds__(256) void k_hist(const void* payload, Geom g, const QParam* qp, uint32_t* hist,
                                              uint32_t bpt) {
    extern __shared__ __align__(16) uint32_t lh[];
    const uint32_t t = blockIdx.x / bpt, b = blockIdx.x % bpt;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    HistLds H;
    H.win_bins = hist_win_bins(g.K);
    H.win_lo = g.R - H.win_bins / 2u;  // symbol R is the bin of value 0
    const uint32_t n_words = H.win_bins * kHistCopies + g.K + kW;
    H.ovf_byte = H.win_bins * kHistCopies * 4u;
    H.trash_byte = (H.win_bins * kHistCopies + g.K + lane) * 4u;
    for (uint32_t k = tid; k < n_words; k += 256) lh[k] = 0;
    __syncthreads();
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t turns = g.S / kV;
    for (uint32_t grp = b * 4 + wave; grp < g.G; grp += bpt * 4) {
        const uint32_t gstart = grp * (kW * g.S);
        const uint8_t* gbase = tab + (size_t)gstart * g.es;
        const uint32_t rem = g.n - gstart;
        if (rem >= kW * g.S) hist_group<F16, VEC, true>(gbase, rem, turns, lane, q, Rf, (int)g.R, lh, H);
        else hist_group<F16, VEC, false>(gbase, rem, turns, lane, q, Rf, (int)g.R, lh, H);
    }
    __syncthreads();
    // merge: window bins (sum of the copies, skewed start so that the threads of a wavefront read different
    // banks) plus the overflow array
    const uint32_t* ovf = lh + H.win_bins * kHistCopies;
    for (uint32_t k = tid; k < g.K; k += 256) {
        uint32_t s = ovf[k];
        const uint32_t w = k - H.win_lo;
        if (w < H.win_bins) {
            const uint32_t* row = lh + w * kHistCopies;
            for (uint32_t c = 0; c < kHistCopies; ++c) s += row[(c + tid) & (kHistCopies - 1u)];
        }
        if (s) atomicAdd(&hist[(size_t)t * g.K + k], s);
    }
}

// ------------------------------------------------------------------------------------------------
// Huffman codebook of one table, built by one work-group of 256 threads from the table's histogram.
//   leaves ordered by (count, symbol); two queues (leaves, merged nodes in creation order); a tie
//   between the queue heads takes the leaf; longest code above LMAX: lengths are cut to LMAX, the
//   Kraft sum is repaired one unit at a time (a code of length LMAX pairs up with a code taken from
//   the deepest shorter level) and the resulting lengths are handed out most frequent symbol first;
//   canonical codewords in (length, symbol) order.  One used symbol: length 0.
//   smem: codebook_smem(K) bytes, 16-byte aligned.  Ends with a barrier; results are in global memory.
// ------------------------------------------------------------------------------------------------
__host__ __device__ constexpr size_t codebook_smem(uint32_t K) { return (size_t)K * (8 + 4 + 4 + 2 + 2 + 2 + 2) + 64 * 4; }

struct CodebookShared {
    uint32_t lo, hi, maxlen, cl[kLmaxLimit + 2], next[kLmaxLimit + 2];
};

// hist_t is read, copied to hist_view_t (inspection) and cleared, so that the next call starts from zero counts.
__device__ __forceinline__ void codebook_build(const Geom& g, uint32_t* hist_t, uint32_t* hist_view_t, uint16_t* enc_t,
                                               uint8_t* lens_t, TMeta* tmeta_t, unsigned char* smem, CodebookShared& sh,
                                               uint32_t tid) {
    const uint32_t K = g.K;
    uint64_t* key = reinterpret_cast<uint64_t*>(smem);        // [K] sort keys: count << 16 | symbol
    uint32_t* cnt = reinterpret_cast<uint32_t*>(key + K);      // [K] counts
    uint32_t* nodew = cnt + K;                                 // [K] merged-node weights, later codewords
    uint16_t* parent_leaf = reinterpret_cast<uint16_t*>(nodew + K);  // [K] parent of a leaf, later its length
    uint16_t* parent_node = parent_leaf + K;                   // [K]
    uint16_t* depth_node = parent_node + K;                    // [K]
    uint16_t* len_s = depth_node + K;                          // [K] code length per symbol
    uint32_t* scratch = reinterpret_cast<uint32_t*>(len_s + K);  // [64]

    DLC_STAMP(0);
    for (uint32_t k = tid; k < K; k += 256) {
        const uint32_t h = hist_t[k];
        cnt[k] = h;
        hist_view_t[k] = h;
        hist_t[k] = 0;
        len_s[k] = 0;
    }
    if (tid == 0) { sh.lo = 0xFFFFFFFFu; sh.hi = 0; sh.maxlen = 0; }
    if (tid < kLmaxLimit + 2) sh.cl[tid] = 0;
    __syncthreads();

    // compaction offsets of the used symbols (symbol order)
    const uint32_t per = (K + 255) / 256;
    const uint32_t k0 = tid * per, k1 = min(K, k0 + per);
    uint32_t mine = 0;
    for (uint32_t k = k0; k < k1; ++k) mine += cnt[k] != 0;
    uint32_t n_used;
    const uint32_t my_off = block_excl_scan<4>(mine, scratch, tid, &n_used);
    for (uint32_t k = k0; k < k1; ++k)
        if (cnt[k]) { atomicMin(&sh.lo, k); atomicMax(&sh.hi, k); }
    __syncthreads();

    DLC_STAMP(1);
    if (n_used >= 2) {
        uint32_t P = 2;
        while (P < n_used) P <<= 1;
        // keys of the used symbols, padded to a power of two
        {
            uint32_t o = my_off;
            for (uint32_t k = k0; k < k1; ++k)
                if (cnt[k]) key[o++] = ((uint64_t)cnt[k] << 16) | k;
            for (uint32_t i = n_used + tid; i < P; i += 256) key[i] = ~0ull;
        }
        __syncthreads();
        DLC_STAMP(2);
        // bitonic sort, ascending
        for (uint32_t size = 2; size <= P; size <<= 1) {
            for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
                for (uint32_t i = tid; i < (P >> 1); i += 256) {
                    uint32_t lo = 2 * i - (i & (stride - 1));
                    uint32_t hi = lo + stride;
                    bool up = (lo & size) == 0;
                    uint64_t a = key[lo], bb = key[hi];
                    if ((a > bb) == up) { key[lo] = bb; key[hi] = a; }
                }
                __syncthreads();
            }
        }
        DLC_STAMP(3);
        if (tid == 0) {
            const uint32_t n = n_used;
            uint32_t a = 0, bq = 0;  // heads of the leaf queue and of the merged-node queue
            for (uint32_t k = 0; k + 1 < n; ++k) {
                uint32_t sum = 0;
                for (int pick = 0; pick < 2; ++pick) {
                    bool take_leaf;
                    if (a >= n) take_leaf = false;
                    else if (bq >= k) take_leaf = true;
                    else take_leaf = (uint32_t)(key[a] >> 16) <= nodew[bq];
                    if (take_leaf) { sum += (uint32_t)(key[a] >> 16); parent_leaf[a] = (uint16_t)k; ++a; }
                    else { sum += nodew[bq]; parent_node[bq] = (uint16_t)k; ++bq; }
                }
                nodew[k] = sum;
            }
            depth_node[n - 2] = 0;
            for (int k = (int)n - 3; k >= 0; --k) depth_node[k] = depth_node[parent_node[k]] + 1;
            sh.maxlen = 0;
        }
        __syncthreads();
        DLC_STAMP(4);
        // leaf depths; parent_leaf[] is reused to hold the depth of leaf i (sorted order)
        uint32_t local_max = 0;
        for (uint32_t i = tid; i < n_used; i += 256) {
            const uint32_t d = depth_node[parent_leaf[i]] + 1u;
            parent_leaf[i] = (uint16_t)d;
            local_max = max(local_max, d);
        }
        if (local_max) atomicMax(&sh.maxlen, local_max);
        __syncthreads();
        if (sh.maxlen > g.LMAX) {
            for (uint32_t i = tid; i < n_used; i += 256) atomicAdd(&sh.cl[min((uint32_t)parent_leaf[i], g.LMAX)], 1u);
            __syncthreads();
            if (tid == 0) {
                const uint32_t LM = g.LMAX;
                uint64_t kraft = 0;
                for (uint32_t L = 1; L <= LM; ++L) kraft += (uint64_t)sh.cl[L] << (LM - L);
                while (kraft > (1ull << LM) && sh.cl[LM] > 0) {
                    sh.cl[LM] -= 1;
                    for (uint32_t L = LM - 1; L >= 1; --L)
                        if (sh.cl[L]) { sh.cl[L] -= 1; sh.cl[L + 1] += 2; break; }
                    kraft -= 1;
                }
                // next[L] = number of leaves (counted from the most frequent) with length < L
                uint32_t acc = 0;
                for (uint32_t L = 1; L <= LM; ++L) { sh.next[L] = acc; acc += sh.cl[L]; }
                sh.next[LM + 1] = acc;
            }
            __syncthreads();
            for (uint32_t i = tid; i < n_used; i += 256) {
                const uint32_t rank = n_used - 1u - i;  // 0 = most frequent (leaves are sorted by rising count)
                uint32_t L = 1;
                while (L < g.LMAX && rank >= sh.next[L + 1]) ++L;
                parent_leaf[i] = (uint16_t)L;
            }
            __syncthreads();
            if (tid < kLmaxLimit + 2) sh.cl[tid] = 0;
            __syncthreads();
        }
        for (uint32_t i = tid; i < n_used; i += 256) len_s[(uint32_t)(key[i] & 0xFFFFu)] = parent_leaf[i];
        __syncthreads();
        // codewords
        DLC_STAMP(5);
        for (uint32_t k = k0; k < k1; ++k)
            if (len_s[k]) atomicAdd(&sh.cl[len_s[k]], 1u);
        __syncthreads();
        if (tid == 0) {
            uint32_t code = 0;
            for (uint32_t L = 1; L <= g.LMAX; ++L) {
                code <<= 1;
                sh.next[L] = code;
                code += sh.cl[L];
            }
            for (uint32_t k = sh.lo; k <= sh.hi; ++k) {
                uint32_t L = len_s[k];
                if (L) nodew[k] = sh.next[L]++;
            }
        }
        __syncthreads();
    }
    DLC_STAMP(6);
    for (uint32_t k = tid; k < K; k += 256) {
        uint32_t L = len_s[k];
        enc_t[k] = (uint16_t)(L ? ((L << 12) | nodew[k]) : 0u);
        lens_t[k] = (uint8_t)L;
    }
    if (tid == 0) {
        TMeta m;
        // an empty histogram cannot come out of the histogram kernel (every table has an element); should it
        // happen anyway, the symbol range must still be a valid one for the kernels that size things from it
        if (n_used == 0) { sh.lo = 0; sh.hi = 0; }
        m.n_used = n_used; m.sym_lo = sh.lo; m.sym_hi = sh.hi; m.n_outliers = cnt[0];  // symbol 0 = escape
        m.cb_off = 0; m.outl_off = 0;
        *tmeta_t = m;
    }
    __syncthreads();
    DLC_STAMP(7);
}

__global__ __launch_bounds__(256) void k_codebook(Geom g, uint32_t* hist, uint32_t* hist_view, uint16_t* enc,
                                                  uint8_t* lens, TMeta* tmeta) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ CodebookShared sh;
    const uint32_t t = blockIdx.x;
    codebook_build(g, hist + (size_t)t * g.K, hist_view + (size_t)t * g.K, enc + (size_t)t * g.K,
                   lens + (size_t)t * g.K, tmeta + t, smem, sh, threadIdx.x);
}

// ------------------------------------------------------------------------------------------------
// bit-packed encode.
//   walk 1: load, quantise, look the (length, codeword) pairs up in LDS, keep them packed in registers,
//           sum the chunk's bits, count the escapes
//   scan  : chunk word counts inside the wavefront; group totals (chunk words + two words per escape)
//           across the grid by a single-pass look-back over per-group records (ordered work-group ids:
//           a group only ever waits for groups of work-groups that started earlier)
//   walk 2: shift the kept pairs into a 64-bit accumulator, store whole words at the chunk's offset
//   escapes (rare for fp32): a group that has any walks its elements once more in a rolled loop and
//           writes its records, in increasing element index, behind its chunk words
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kFlagAgg = 1, kFlagPrefix = 2;
constexpr uint32_t kSpinLimit = 1u << 22;

// exclusive prefix of `total` over all groups before gid; publishes this group's records.  All lanes call.
__device__ __forceinline__ uint32_t group_scan(uint64_t* state, uint64_t epoch, uint32_t gid, uint32_t total,
                                               uint32_t lane, Ctrl* ctrl, bool* dead) {
    const uint64_t tag = epoch << 34;
    if (lane == 0)
        __hip_atomic_store(&state[gid], tag | ((uint64_t)(gid == 0 ? kFlagPrefix : kFlagAgg) << 32) | total,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t excl = 0;
    if (gid > 0) {
        int64_t pos = (int64_t)gid - 1;
        uint32_t spins = 0;
        for (;;) {
            const int64_t my = pos - (int64_t)lane;
            uint64_t sv;
            uint32_t flag;
            for (;;) {
                sv = my >= 0 ? __hip_atomic_load(&state[my], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                             : (tag | ((uint64_t)kFlagPrefix << 32));
                flag = (sv >> 34) == epoch ? (uint32_t)(sv >> 32) & 3u : 0u;
                if (__ballot(flag == 0u) == 0ull) break;
                if (++spins > kSpinLimit) break;  // never expected; the bound only guarantees termination
                __builtin_amdgcn_s_sleep(2);
            }
            if (spins > kSpinLimit) {
                if (lane == 0) { set_status(ctrl, DLC_ESTATE); ctrl->abort = 1; }
                *dead = true;
                break;
            }
            const uint64_t pm = __ballot(flag == kFlagPrefix);
            if (pm) {
                const uint32_t first = (uint32_t)__ffsll((unsigned long long)pm) - 1u;
                excl += wave_sum(lane <= first ? (uint32_t)sv : 0u);
                break;
            }
            excl += wave_sum((uint32_t)sv);
            pos -= 64;
        }
        if (lane == 0)
            __hip_atomic_store(&state[gid], tag | ((uint64_t)kFlagPrefix << 32) | (uint32_t)(excl + total),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return excl;
}

// walk 2 and everything after the group's offset is known.  pk[] holds S/2 words of two (len<<12|code) each.
template <int S, bool F16, bool VEC>
__device__ __forceinline__ void emit_group(const uint32_t (&pk)[S / 2], uint32_t nw, uint32_t lane_off, uint32_t excl,
                                           uint32_t chunk_total, uint32_t n_esc, uint32_t gid, uint32_t lane,
                                           const uint8_t* gbase, uint32_t gstart, uint32_t rem, const QParam& q, float Rf,
                                           int R, const FixedLayout& F, uint8_t* out) {
    out[F.off_chunk + (uint64_t)gid * kW + lane] = (uint8_t)nw;
    if (lane == 0) reinterpret_cast<uint32_t*>(out + F.off_group)[gid] = excl;
    uint32_t* gw = reinterpret_cast<uint32_t*>(out + F.off_payload) + excl;
    uint32_t* p = gw + lane_off;
    uint64_t acc = 0;
    uint32_t nb = 0;
#pragma clang loop unroll(full)
    for (int i = 0; i < S / 2; ++i) {
        const uint32_t w = pk[i];
        const uint32_t l0 = (w >> 12) & 0xFu, l1 = w >> 28;
        acc = (acc << l0) | (w & 0xFFFu);
        acc = (acc << l1) | ((w >> 16) & 0xFFFu);
        nb += l0 + l1;
        if (nb >= 32u) {
            nb -= 32u;
            *p++ = (uint32_t)(acc >> nb);
        }
        if ((i & 3) == 3) __builtin_amdgcn_sched_barrier(0);  // do not unpack far ahead of the serial chain
    }
    if (nb) *p = (uint32_t)(acc << (32u - nb));
    if (n_esc != 0u) {  // uniform over the wavefront
        uint32_t* rec = gw + chunk_total;
        uint32_t opos = 0;
        for (uint32_t j = 0; j < (uint32_t)S / kV; ++j) {
            const uint32_t off = lane * kV + j * (kW * kV);
            float x[4];
            uint32_t raw[4];
            const uint32_t valid = load4<F16, VEC>(gbase, off, rem, x, raw);
            uint32_t esc = 0;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                esc |= (((valid >> v) & 1u) && quant_symbol<F16>(x[v], q, Rf, R) == 0u) ? (1u << v) : 0u;
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
}

template <int S, bool F16, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(S == 256 ? 2 : (S == 128 ? 3 : 5))))
void k_encode(const void* payload, Geom g, FixedLayout F, const QParam* qp, const uint16_t* enc, Ctrl* ctrl,
              uint64_t* state, uint64_t epoch, uint8_t* out, uint64_t capacity, uint32_t bpt, uint32_t* word_start,
              uint32_t* word_end) {
    extern __shared__ __align__(16) uint16_t s_enc[];
    __shared__ uint32_t s_wg;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    if (tid == 0) s_wg = atomicAdd(&ctrl->ticket, 1u);
    __syncthreads();
    const uint32_t wg = __builtin_amdgcn_readfirstlane(s_wg);
    const uint32_t t = wg / bpt, b = wg % bpt;
    for (uint32_t k = tid; k < g.K; k += 256) s_enc[k] = enc[(size_t)t * g.K + k];
    __syncthreads();
    const uint32_t grp = b * 4 + __builtin_amdgcn_readfirstlane(wave);
    if (grp >= g.G) return;  // whole wavefront; no barrier follows
    const uint32_t gid = t * g.G + grp;
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    bool dead = false;  // nothing may be written to the container
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t gstart = grp * (kW * (uint32_t)S);
    const uint8_t* gbase = tab + (size_t)gstart * g.es;
    const uint32_t rem = g.n - gstart;

    uint32_t pk[S / 2];
    uint32_t bits = 0;
    uint32_t n_esc = 0;  // escapes of the whole group (a scalar: counted from the comparison masks)
    constexpr int kBlk = 8;  // turns whose loads are in flight together (8 x 16 B per lane)
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
            uint32_t e[4];
#pragma clang loop unroll(full)
            for (int v = 0; v < 4; ++v) {
                const uint32_t c = quant_symbol<F16>(x[u][v], q, Rf, (int)g.R);
                const bool ok = (valid[u] >> v) & 1u;
                // unconditional table read, masked afterwards: a position past the end contributes no bits
                e[v] = (uint32_t)s_enc[c] & (0u - (uint32_t)ok);
                n_esc += (uint32_t)__popcll(__ballot(ok && c == 0u));
            }
            uint32_t w0 = e[0] | (e[1] << 16), w1 = e[2] | (e[3] << 16);
            // opaque to the optimiser: otherwise it keeps length and codeword of every symbol in registers of
            // their own instead of the packed words
            asm volatile("" : "+v"(w0), "+v"(w1));
            pk[2 * (jb + u)] = w0;
            pk[2 * (jb + u) + 1] = w1;
            bits += ((w0 >> 12) & 0xFu) + (w0 >> 28) + ((w1 >> 12) & 0xFu) + (w1 >> 28);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the next block's loads from being hoisted above this one
    }
    const uint32_t nw = (bits + 31u) >> 5;
    const uint32_t incl = wave_incl_scan(nw, lane);
    const uint32_t lane_off = incl - nw;
    const uint32_t chunk_total = __shfl(incl, 63, 64);
    const uint32_t total = chunk_total + 2u * n_esc;

    const uint32_t excl = group_scan(state, epoch, gid, total, lane, ctrl, &dead);
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
}

// ------------------------------------------------------------------------------------------------
// finalize: code-length blocks behind the payload, header, directory, padding, size metadata; clears the
// per-call control words for the next call.  One work-group of 1024 threads.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t a16(uint64_t x) { return (x + 15ull) & ~15ull; }

__global__ __launch_bounds__(1024) void k_finalize(Geom g, FixedLayout F, const TMeta* tmeta, const uint8_t* __restrict__ lens,
                                                   const QParam* qp, Ctrl* ctrl, const uint32_t* word_start,
                                                   const uint32_t* word_end, uint8_t* __restrict__ out, uint64_t capacity,
                                                   uint64_t* out_bytes) {
    __shared__ uint32_t s_red[17];
    __shared__ uint32_t s_abort;
    __shared__ uint32_t s_cb[1025];   // start of each table's block, relative to the pass's first block
    __shared__ uint32_t s_lo[1024], s_nl[1024];
    const uint32_t tid = threadIdx.x;
    const uint64_t words = word_end[g.T - 1];
    const uint64_t off_cb = a16(F.off_payload + 4ull * words);
    const bool aborted = ctrl->abort != 0;
    uint64_t cb_carry = 0, nout_carry = 0;
    for (uint32_t base = 0; base < g.T; base += 1024) {
        const uint32_t t = base + tid;
        TMeta m;
        uint32_t cb = 0, no = 0, nl = 0;
        if (t < g.T) {
            m = tmeta[t];
            if (m.sym_lo > m.sym_hi || m.sym_hi >= g.K) { m.sym_lo = 0; m.sym_hi = 0; }  // never index outside lens[]
            nl = m.sym_hi - m.sym_lo + 1u;
            cb = (nl + 3u) & ~3u;
            no = m.n_outliers;
        }
        uint32_t cb_tot, no_tot;
        const uint32_t cb_ex = block_excl_scan<16>(cb, s_red, tid, &cb_tot);
        __syncthreads();
        (void)block_excl_scan<16>(no, s_red, tid, &no_tot);
        s_cb[tid] = cb_ex;
        s_lo[tid] = m.sym_lo;
        s_nl[tid] = nl;
        if (tid == 0) {
            s_cb[1024] = cb_tot;
            // the code-length blocks are the last thing in the container: the capacity check of this pass
            s_abort = aborted || off_cb + cb_carry + cb_tot > capacity;
        }
        __syncthreads();
        if (s_abort) break;  // uniform
        const uint32_t nt = min(1024u, g.T - base);
        // the pass's blocks, byte by byte: binary search for the table of byte j
        for (uint32_t j = tid; j < cb_tot; j += 1024) {
            uint32_t lo = 0, hi = nt - 1u;
            while (lo < hi) {
                const uint32_t mid = (lo + hi + 1u) >> 1;
                if (s_cb[mid] <= j) lo = mid; else hi = mid - 1u;
            }
            const uint32_t i = j - s_cb[lo];
            out[off_cb + cb_carry + j] = i < s_nl[lo] ? lens[(size_t)(base + lo) * g.K + s_lo[lo] + i] : (uint8_t)0;
        }
        if (t < g.T) {
            const uint64_t w0 = word_start[t], w1 = word_end[t];
            uint8_t* d = out + kHeaderBytes + (uint64_t)kDirBytes * t;
            uint32_t* d32 = reinterpret_cast<uint32_t*>(d);
            d32[0] = qp[t].eb_bits; d32[1] = m.n_used; d32[2] = m.sym_lo; d32[3] = m.sym_hi; d32[4] = m.n_outliers;
            d32[5] = g.G;
            uint64_t* d64 = reinterpret_cast<uint64_t*>(d + 24);
            d64[0] = off_cb + cb_carry + cb_ex; d64[1] = 0; d64[2] = w0; d64[3] = w1 - w0;
            out_bytes[1 + t] = 4ull * (w1 - w0) + cb + (uint64_t)(kW + 4u) * g.G + kDirBytes;
        }
        cb_carry += cb_tot;
        nout_carry += no_tot;
        __syncthreads();
    }
    if (s_abort) {
        if (tid == 0 && !aborted) set_status(ctrl, DLC_ECAPACITY);
        for (uint32_t t = tid; t < g.T + 1; t += 1024) out_bytes[t] = 0;
    } else {
        // padding between sections
        const uint64_t e0 = kHeaderBytes + (uint64_t)kDirBytes * g.T;
        for (uint64_t i = e0 + tid; i < F.off_group; i += 1024) out[i] = 0;
        const uint64_t e1 = F.off_group + 4ull * g.NG;
        for (uint64_t i = e1 + tid; i < F.off_chunk; i += 1024) out[i] = 0;
        const uint64_t e2 = F.off_payload + 4ull * words;
        for (uint64_t i = e2 + tid; i < off_cb; i += 1024) out[i] = 0;
        if (tid == 0) {
            uint32_t* h = reinterpret_cast<uint32_t*>(out);
            h[H_MAGIC] = kMagic; h[H_VERSION] = kVersion; h[H_DTYPE] = g.dtype; h[H_T] = g.T; h[H_B] = g.B; h[H_D] = g.D;
            h[H_R] = g.R; h[H_S] = g.S; h[H_LMAX] = g.LMAX; h[H_W] = kW; h[H_V] = kV; h[H_NG] = g.NG;
            uint64_t* q = reinterpret_cast<uint64_t*>(out);
            q[HQ_NOUT] = nout_carry; q[HQ_WORDS] = words; q[HQ_OFF_GROUP] = F.off_group; q[HQ_OFF_CHUNK] = F.off_chunk;
            q[HQ_OFF_PAYLOAD] = F.off_payload; q[HQ_OFF_CB] = off_cb;
            const uint64_t total = off_cb + cb_carry;
            q[HQ_TOTAL] = total; q[HQ_TOTAL + 1] = 0; q[HQ_TOTAL + 2] = 0; q[HQ_TOTAL + 3] = 0;
            out_bytes[0] = total;
        }
    }
    // the next call starts with ticket 0 and no abort (the histograms were cleared by the codebook step)
    if (tid == 0) { ctrl->ticket = 0; ctrl->abort = 0; }
}

// ------------------------------------------------------------------------------------------------
template <int S>
static void launch_encode_s(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch,
                            uint8_t* out, uint64_t capacity, uint32_t bpt, hipStream_t s) {
    dim3 grid(g.T * bpt), block(256);
    size_t sm = (size_t)g.K * 2;
    const bool f16 = g.dtype == DLC_F16;
#define DLC_ENC(FF, V)                                                                                          \
    hipLaunchKernelGGL((k_encode<S, FF, V>), grid, block, sm, s, payload, g, F, w.qp, w.enc, w.ctrl, w.state, epoch, \
                       out, capacity, bpt, w.word_start, w.word_end)
    if (f16) { if (g.vec) DLC_ENC(true, true); else DLC_ENC(true, false); }
    else { if (g.vec) DLC_ENC(false, true); else DLC_ENC(false, false); }
#undef DLC_ENC
}

hipError_t launch_compress(const Geom& g, const void* payload, uint8_t* out, uint64_t capacity, uint64_t* out_bytes,
                           const Ws& w, uint64_t epoch, int pl, void* prof, hipStream_t s) {
    const bool f16 = g.dtype == DLC_F16;
    const FixedLayout F = fixed_layout(g);
    // histogram
    uint32_t bpt_h = (g.G + 3) / 4;
    {
        // cap the grid at a few work-groups per CU; a work-group then loops over groups of its table
        const uint32_t max_blocks = 256 * 8;
        const uint32_t cap = std::max<uint32_t>(1, max_blocks / g.T);
        bpt_h = std::min(bpt_h, cap);
        const size_t sm = hist_lds_bytes(g.K);
        dim3 grid(g.T * bpt_h), block(256);
        if (prof_on(pl, P_HIST)) prof_begin(prof, P_HIST, s);
#define DLC_HIST(FF, V) hipLaunchKernelGGL((k_hist<FF, V>), grid, block, sm, s, payload, g, w.qp, w.hist, bpt_h)
        if (f16) { if (g.vec) DLC_HIST(true, true); else DLC_HIST(true, false); }
        else { if (g.vec) DLC_HIST(false, true); else DLC_HIST(false, false); }
#undef DLC_HIST
        if (prof_on(pl, P_HIST)) prof_end(prof, P_HIST, s);
    }
    if (prof_on(pl, P_CODEBOOK)) prof_begin(prof, P_CODEBOOK, s);
    hipLaunchKernelGGL(k_codebook, dim3(g.T), dim3(256), codebook_smem(g.K), s, g, w.hist, w.hist_view, w.enc, w.lens,
                       w.tmeta);
    if (prof_on(pl, P_CODEBOOK)) prof_end(prof, P_CODEBOOK, s);
    {
        const uint32_t bpt = (g.G + 3) / 4;
        if (prof_on(pl, P_ENCODE)) prof_begin(prof, P_ENCODE, s);
        switch (g.S) {
            case 64: launch_encode_s<64>(g, F, payload, w, epoch, out, capacity, bpt, s); break;
            case 128: launch_encode_s<128>(g, F, payload, w, epoch, out, capacity, bpt, s); break;
            default: launch_encode_s<256>(g, F, payload, w, epoch, out, capacity, bpt, s); break;
        }
        if (prof_on(pl, P_ENCODE)) prof_end(prof, P_ENCODE, s);
    }
    if (prof_on(pl, P_FINALIZE)) prof_begin(prof, P_FINALIZE, s);
    hipLaunchKernelGGL(k_finalize, dim3(1), dim3(1024), 0, s, g, F, w.tmeta, w.lens, w.qp, w.ctrl, w.word_start,
                       w.word_end, out, capacity, out_bytes);
    if (prof_on(pl, P_FINALIZE)) prof_end(prof, P_FINALIZE, s);
    return hipGetLastError();
}

hipError_t compress_set_attributes() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k_codebook), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)codebook_smem(4096));
}

}  // namespace dlc
