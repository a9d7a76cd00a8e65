// Compression kernels for gfx950: quantise + histogram, Huffman codebook, container layout,
// bit-packed encode with scanned offsets, finalize.
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
// quantise + LDS-privatised histogram + escape counts per group
//   grid: T * bpt work-groups of 4 wavefronts; a work-group stays inside one table
//   LDS : K << clog2 counters; a lane adds into copy (lane & (C-1)) of its bin so that the few hot
//         bins of a bell-shaped distribution spread over C banks instead of serialising on one address
// ------------------------------------------------------------------------------------------------
template <bool F16, bool VEC>
__global__ __launch_bounds__(256) void k_hist(const void* payload, Geom g, const QParam* qp, uint32_t* hist,
                                              uint32_t* group_outliers, uint32_t* table_outliers, uint32_t bpt,
                                              uint32_t clog2) {
    extern __shared__ __align__(16) uint32_t lh[];
    const uint32_t t = blockIdx.x / bpt, b = blockIdx.x % bpt;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t nbins = g.K << clog2;
    for (uint32_t k = tid; k < nbins + kW; k += 256) lh[k] = 0;
    __syncthreads();
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    const uint32_t cm = lane & ((1u << clog2) - 1u);
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t turns = g.S / kV;
    for (uint32_t grp = b * 4 + wave; grp < g.G; grp += bpt * 4) {
        const uint32_t gstart = grp * (kW * g.S);
        const uint8_t* gbase = tab + (size_t)gstart * g.es;
        const uint32_t rem = g.n - gstart;
        uint32_t nout = 0;
#ifndef DLC_EXP_HIST_BLK
#define DLC_EXP_HIST_BLK 4
#endif
        constexpr uint32_t kBlk = DLC_EXP_HIST_BLK;  // turns whose loads are issued back to back (S/4 is a multiple)
        for (uint32_t jb = 0; jb < turns; jb += kBlk) {
            float x[kBlk][4];
            uint32_t raw[kBlk][4];
            uint32_t valid[kBlk];
#pragma unroll
            for (uint32_t u = 0; u < kBlk; ++u)
                valid[u] = load4<F16, VEC>(gbase, lane * kV + (jb + u) * (kW * kV), rem, x[u], raw[u]);
#pragma unroll
            for (uint32_t u = 0; u < kBlk; ++u) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    // branch-free: a position past the end of the table counts into a scratch bin of its own lane
                    const bool ok = (valid[u] >> v) & 1u;
                    const uint32_t c = quant_symbol<F16>(x[u][v], q, Rf, (int)g.R);
                    atomicAdd(&lh[ok ? (c << clog2) + cm : nbins + lane], 1u);
                    nout += (ok && c == 0u) ? 1u : 0u;
                }
            }
        }
        nout = wave_sum(nout);
        if (lane == 0) {
            group_outliers[t * g.G + grp] = nout;
            if (nout) atomicAdd(&table_outliers[t], nout);
        }
    }
    __syncthreads();
    const uint32_t C = 1u << clog2;
    for (uint32_t k = tid; k < g.K; k += 256) {
        uint32_t s = 0;
        for (uint32_t c = 0; c < C; ++c) s += lh[(k << clog2) + c];
        if (s) atomicAdd(&hist[(size_t)t * g.K + k], s);
    }
}

// ------------------------------------------------------------------------------------------------
// Huffman codebook, one work-group per table.
//   leaves ordered by (count, symbol); two queues (leaves, merged nodes in creation order); a tie
//   between the queue heads takes the leaf; longest code d bits above LMAX: every count becomes
//   ceil(count / 2^d) and the tree is rebuilt, until it fits; canonical codewords in (length, symbol)
//   order.  One used symbol: length 0.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_codebook(Geom g, const uint32_t* hist, const uint32_t* table_outliers,
                                                  uint16_t* enc, uint8_t* lens, TMeta* tmeta) {
    extern __shared__ __align__(16) unsigned char smem[];  // the 64-bit sort keys need natural alignment
    const uint32_t K = g.K, tid = threadIdx.x, t = blockIdx.x;
    uint64_t* key = reinterpret_cast<uint64_t*>(smem);        // [K] sort keys: count << 16 | symbol
    uint32_t* cnt = reinterpret_cast<uint32_t*>(key + K);      // [K] working counts
    uint32_t* nodew = cnt + K;                                 // [K] merged-node weights
    uint16_t* parent_leaf = reinterpret_cast<uint16_t*>(nodew + K);  // [K]
    uint16_t* parent_node = parent_leaf + K;                   // [K]
    uint16_t* depth_node = parent_node + K;                    // [K]
    uint16_t* len_s = depth_node + K;                          // [K] code length per symbol
    uint32_t* scratch = reinterpret_cast<uint32_t*>(len_s + K);  // [256]
    __shared__ uint32_t s_lo, s_hi, s_maxlen, s_cl[kLmaxLimit + 2], s_next[kLmaxLimit + 2];

    DLC_STAMP(0);
    for (uint32_t k = tid; k < K; k += 256) {
        cnt[k] = hist[(size_t)t * K + k];
        len_s[k] = 0;
    }
    if (tid == 0) { s_lo = 0xFFFFFFFFu; s_hi = 0; s_maxlen = 0; }
    if (tid < kLmaxLimit + 2) s_cl[tid] = 0;
    __syncthreads();

    // compaction offsets of the used symbols (symbol order)
    const uint32_t per = (K + 255) / 256;
    const uint32_t k0 = tid * per, k1 = min(K, k0 + per);
    uint32_t mine = 0;
    for (uint32_t k = k0; k < k1; ++k) mine += cnt[k] != 0;
    uint32_t n_used;
    const uint32_t my_off = block_excl_scan<4>(mine, scratch, tid, &n_used);
    __syncthreads();
    for (uint32_t k = k0; k < k1; ++k)
        if (cnt[k]) { atomicMin(&s_lo, k); atomicMax(&s_hi, k); }
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
            s_maxlen = 0;
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
        if (local_max) atomicMax(&s_maxlen, local_max);
        __syncthreads();
        if (s_maxlen > g.LMAX) {
            // cut to LMAX, repair the Kraft sum one unit at a time, hand the lengths out most frequent first
            for (uint32_t i = tid; i < n_used; i += 256) atomicAdd(&s_cl[min((uint32_t)parent_leaf[i], g.LMAX)], 1u);
            __syncthreads();
            if (tid == 0) {
                const uint32_t LM = g.LMAX;
                uint64_t kraft = 0;
                for (uint32_t L = 1; L <= LM; ++L) kraft += (uint64_t)s_cl[L] << (LM - L);
                while (kraft > (1ull << LM)) {
                    s_cl[LM] -= 1;
                    for (uint32_t L = LM - 1; L >= 1; --L)
                        if (s_cl[L]) { s_cl[L] -= 1; s_cl[L + 1] += 2; break; }
                    kraft -= 1;
                }
                // s_next[L] = number of leaves (counted from the most frequent) with length < L
                uint32_t acc = 0;
                for (uint32_t L = 1; L <= LM; ++L) { s_next[L] = acc; acc += s_cl[L]; }
                s_next[LM + 1] = acc;
            }
            __syncthreads();
            for (uint32_t i = tid; i < n_used; i += 256) {
                const uint32_t rank = n_used - 1u - i;  // 0 = most frequent (leaves are sorted by rising count)
                uint32_t L = 1;
                while (rank >= s_next[L + 1]) ++L;
                parent_leaf[i] = (uint16_t)L;
            }
            __syncthreads();
            if (tid < kLmaxLimit + 2) s_cl[tid] = 0;
            __syncthreads();
        }
        for (uint32_t i = tid; i < n_used; i += 256) len_s[(uint32_t)(key[i] & 0xFFFFu)] = parent_leaf[i];
        __syncthreads();
        // codewords
        DLC_STAMP(5);
        for (uint32_t k = k0; k < k1; ++k)
            if (len_s[k]) atomicAdd(&s_cl[len_s[k]], 1u);
        __syncthreads();
        if (tid == 0) {
            uint32_t code = 0;
            for (uint32_t L = 1; L <= g.LMAX; ++L) {
                code <<= 1;
                s_next[L] = code;
                code += s_cl[L];
            }
            for (uint32_t k = s_lo; k <= s_hi; ++k) {
                uint32_t L = len_s[k];
                if (L) nodew[k] = s_next[L]++;  // nodew reused: codeword per symbol
            }
        }
        __syncthreads();
    }
    DLC_STAMP(6);
    for (uint32_t k = tid; k < K; k += 256) {
        uint32_t L = len_s[k];
        enc[(size_t)t * K + k] = (uint16_t)(L ? ((L << 12) | nodew[k]) : 0u);
        lens[(size_t)t * K + k] = (uint8_t)L;
    }
    if (tid == 0) {
        TMeta m;
        m.n_used = n_used; m.sym_lo = s_lo; m.sym_hi = s_hi; m.n_outliers = table_outliers[t];
        m.cb_off = 0; m.outl_off = 0;
        tmeta[t] = m;
    }
    DLC_STAMP(7);
}

static size_t codebook_smem(uint32_t K) { return (size_t)K * (8 + 4 + 4 + 2 + 2 + 2 + 2) + 256 * 4; }

// ------------------------------------------------------------------------------------------------
// container layout: section offsets, scanned escape offsets, header, directory, code lengths
//   one work-group of 1024 threads
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t a16(uint64_t x) { return (x + 15ull) & ~15ull; }

__global__ __launch_bounds__(1024) void k_layout(Geom g, TMeta* tmeta, const uint32_t* group_outliers,
                                                 uint32_t* group_out_base, const uint8_t* lens, const QParam* qp,
                                                 uint8_t* out, uint64_t capacity, Ctrl* ctrl, Layout* lay) {
    __shared__ Layout s_lay;
    __shared__ uint32_t s_red[17];
    __shared__ uint32_t s_abort;
    const uint32_t tid = threadIdx.x;
    // per-table offsets of the code-length blocks and of the escape records: two prefix sums over the tables
    const uint64_t off_cb = a16(kHeaderBytes + (uint64_t)kDirBytes * g.T);
    uint64_t cb_carry = 0, out_carry = 0;
    for (uint32_t base = 0; base < g.T; base += 1024) {
        const uint32_t t = base + tid;
        uint32_t cb = 0, no = 0;
        if (t < g.T) {
            cb = (tmeta[t].sym_hi - tmeta[t].sym_lo + 1u + 3u) & ~3u;
            no = tmeta[t].n_outliers;
        }
        uint32_t cb_tot, no_tot;
        const uint32_t cb_ex = block_excl_scan<16>(cb, s_red, tid, &cb_tot);
        __syncthreads();
        const uint32_t no_ex = block_excl_scan<16>(no, s_red, tid, &no_tot);
        __syncthreads();
        if (t < g.T) {
            tmeta[t].cb_off = off_cb + cb_carry + cb_ex;
            tmeta[t].outl_off = out_carry + no_ex;  // record index for now; byte offset below
        }
        cb_carry += cb_tot;
        out_carry += no_tot;
    }
    if (tid == 0) {
        s_lay.off_cb = off_cb;
        s_lay.off_group = a16(off_cb + cb_carry);
        s_lay.off_chunk = a16(s_lay.off_group + 4ull * g.NG);
        s_lay.off_outl = a16(s_lay.off_chunk + (uint64_t)kW * g.NG);
        s_lay.n_out_total = out_carry;
        s_lay.off_payload = a16(s_lay.off_outl + 8ull * out_carry);
        *lay = s_lay;
        s_abort = s_lay.off_payload > capacity;
        if (s_abort) { ctrl->abort = 1; set_status(ctrl, DLC_ECAPACITY); }
    }
    __syncthreads();
    for (uint32_t t = tid; t < g.T; t += 1024) tmeta[t].outl_off = s_lay.off_outl + 8ull * tmeta[t].outl_off;
    // exclusive prefix sum of the per-group escape counts (all tables, group order)
    uint32_t carry = 0;
    for (uint32_t base = 0; base < g.NG; base += 1024) {
        const uint32_t i = base + tid;
        const uint32_t v = i < g.NG ? group_outliers[i] : 0u;
        uint32_t tot;
        const uint32_t ex = block_excl_scan<16>(v, s_red, tid, &tot);
        __syncthreads();
        if (i < g.NG) group_out_base[i] = carry + ex;
        carry += tot;
    }
    __syncthreads();
    if (s_abort) return;
    // everything before the group-offset section starts as zero (header reserve, padding)
    {
        uint4* z = reinterpret_cast<uint4*>(out);
        const uint64_t n16 = s_lay.off_group / 16;
        for (uint64_t i = tid; i < n16; i += 1024) z[i] = make_uint4(0, 0, 0, 0);
        // the two pads after the group-offset and escape sections
        const uint64_t e1 = s_lay.off_group + 4ull * g.NG;
        for (uint64_t i = e1 + tid; i < s_lay.off_chunk; i += 1024) out[i] = 0;
        const uint64_t e2 = s_lay.off_outl + 8ull * s_lay.n_out_total;
        for (uint64_t i = e2 + tid; i < s_lay.off_payload; i += 1024) out[i] = 0;
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t* h = reinterpret_cast<uint32_t*>(out);
        h[H_MAGIC] = kMagic; h[H_VERSION] = kVersion; h[H_DTYPE] = g.dtype; h[H_T] = g.T; h[H_B] = g.B; h[H_D] = g.D;
        h[H_R] = g.R; h[H_S] = g.S; h[H_LMAX] = g.LMAX; h[H_W] = kW; h[H_V] = kV; h[H_NG] = g.NG;
        uint64_t* q = reinterpret_cast<uint64_t*>(out);
        q[HQ_NOUT] = s_lay.n_out_total;
        q[HQ_OFF_CB] = s_lay.off_cb; q[HQ_OFF_GROUP] = s_lay.off_group; q[HQ_OFF_CHUNK] = s_lay.off_chunk;
        q[HQ_OFF_OUTL] = s_lay.off_outl; q[HQ_OFF_PAYLOAD] = s_lay.off_payload;
        // HQ_WORDS and HQ_TOTAL are filled by k_finalize
    }
    for (uint32_t t = tid; t < g.T; t += 1024) {
        uint8_t* d = out + kHeaderBytes + (uint64_t)kDirBytes * t;
        uint32_t* d32 = reinterpret_cast<uint32_t*>(d);
        const TMeta m = tmeta[t];
        d32[0] = qp[t].eb_bits; d32[1] = m.n_used; d32[2] = m.sym_lo; d32[3] = m.sym_hi; d32[4] = m.n_outliers;
        d32[5] = g.G;
        uint64_t* d64 = reinterpret_cast<uint64_t*>(d + 24);
        d64[0] = m.cb_off; d64[1] = m.outl_off;  // payload offset and size: k_finalize
    }
    // code lengths of the used symbol range: a few dozen bytes per table, one thread per table
    for (uint32_t t = tid; t < g.T; t += 1024) {
        const TMeta m = tmeta[t];
        const uint32_t nl = m.sym_hi - m.sym_lo + 1u;
        const uint8_t* src = lens + (size_t)t * g.K + m.sym_lo;
        for (uint32_t i = 0; i < nl; ++i) out[m.cb_off + i] = src[i];
    }
}

// ------------------------------------------------------------------------------------------------
// bit-packed encode.
//   walk 1: load, quantise, look the (length, codeword) pairs up in LDS, keep them packed in registers,
//           sum the chunk's bits; escapes are written at their scanned positions
//   scan  : chunk word counts inside the wavefront; group totals across the grid by a single-pass
//           look-back over per-group records (ordered work-group ids: a group only ever waits for
//           groups of work-groups that started earlier)
//   walk 2: shift the kept pairs into a 64-bit accumulator, store whole words at the chunk's offset
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kFlagAgg = 1, kFlagPrefix = 2;
constexpr uint32_t kSpinLimit = 1u << 22;

template <int S, bool F16, bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(S == 256 ? 2 : (S == 128 ? 3 : 5))))
void k_encode(const void* payload, Geom g, const QParam* qp, const uint16_t* enc,
                                                const uint32_t* group_outliers, const uint32_t* group_out_base,
                                                const Layout* lay, Ctrl* ctrl,
                                                uint64_t* state, uint64_t epoch, uint8_t* out, uint64_t capacity,
                                                uint32_t bpt, uint32_t* word_start, uint32_t* word_end) {
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
    const Layout L = *lay;
    bool dead = ctrl->abort != 0;  // nothing may be written to the container
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t gstart = grp * (kW * (uint32_t)S);
    const uint8_t* gbase = tab + (size_t)gstart * g.es;
    const uint32_t rem = g.n - gstart;

    uint32_t pk[S / 2];
    uint32_t bits = 0;
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
                // unconditional table read, masked afterwards: a position past the end contributes no bits
                e[v] = (uint32_t)s_enc[c] & (0u - ((valid[u] >> v) & 1u));
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
    // escapes (rare for fp32): the histogram pass counted them per group; a group that has any walks its
    // elements once more in a rolled loop and writes the records in increasing element index
    if (group_outliers[gid] != 0u && !dead) {
        uint32_t opos = group_out_base[gid];
        uint32_t* rec = reinterpret_cast<uint32_t*>(out + L.off_outl);
        for (uint32_t j = 0; j < (uint32_t)S / kV; ++j) {
            const uint32_t off = lane * kV + j * (kW * kV);
            const uint32_t idx = gstart + off;
            float x[4];
            uint32_t raw[4];
            const uint32_t valid = load4<F16, VEC>(gbase, off, rem, x, raw);
            uint32_t esc = 0;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                esc |= (((valid >> v) & 1u) && quant_symbol<F16>(x[v], q, Rf, (int)g.R) == 0u) ? (1u << v) : 0u;
            if (__ballot(esc != 0u) == 0ull) continue;
            const uint32_t cnt = __popc(esc);
            const uint32_t incl = wave_incl_scan(cnt, lane);
            uint32_t p = opos + incl - cnt;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if ((esc >> v) & 1u) {
                    rec[2ull * p] = idx + v;
                    rec[2ull * p + 1] = raw[v];
                    ++p;
                }
            opos += __shfl(incl, 63, 64);
        }
    }
    const uint32_t nw = (bits + 31u) >> 5;
    const uint32_t incl = wave_incl_scan(nw, lane);
    const uint32_t lane_off = incl - nw;
    const uint32_t total = __shfl(incl, 63, 64);

    // ---- offset of this group among all groups --------------------------------------------------
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
                dead = true;
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
    if (L.off_payload + 4ull * ((uint64_t)excl + total) > capacity) {
        if (!dead && lane == 0) { set_status(ctrl, DLC_ECAPACITY); ctrl->abort = 1; }
        dead = true;
    }
    if (lane == 0) {
        if (grp == 0) word_start[t] = excl;
        if (grp == g.G - 1) word_end[t] = excl + total;
    }
    if (dead) return;
    out[L.off_chunk + (uint64_t)gid * kW + lane] = (uint8_t)nw;
    if (lane == 0) reinterpret_cast<uint32_t*>(out + L.off_group)[gid] = excl;

    // ---- walk 2 ----------------------------------------------------------------------------------
    uint32_t* p = reinterpret_cast<uint32_t*>(out + L.off_payload) + excl + lane_off;
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
}

// ------------------------------------------------------------------------------------------------
// sizes: per-table payload extent, totals, size metadata
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_finalize(Geom g, const TMeta* tmeta, const Layout* lay, const Ctrl* ctrl,
                                                  const uint32_t* word_start, const uint32_t* word_end, uint8_t* out,
                                                  uint64_t* out_bytes) {
    const uint32_t tid = threadIdx.x;
    if (ctrl->abort) {
        if (tid == 0) out_bytes[0] = 0;
        for (uint32_t t = tid; t < g.T; t += 256) out_bytes[1 + t] = 0;
        return;
    }
    for (uint32_t t = tid; t < g.T; t += 256) {
        uint64_t* d64 = reinterpret_cast<uint64_t*>(out + kHeaderBytes + (uint64_t)kDirBytes * t + 24);
        const uint64_t w0 = word_start[t], w1 = word_end[t];
        d64[2] = w0;
        d64[3] = w1 - w0;
        const TMeta m = tmeta[t];
        out_bytes[1 + t] = 4ull * (w1 - w0) + ((m.sym_hi - m.sym_lo + 1u + 3u) & ~3u) + 8ull * m.n_outliers +
                           (uint64_t)(kW + 4u) * g.G + kDirBytes;
    }
    if (tid == 0) {
        const uint64_t words = word_end[g.T - 1];
        uint64_t* q = reinterpret_cast<uint64_t*>(out);
        q[HQ_WORDS] = words;
        const uint64_t total = lay->off_payload + 4ull * words;
        q[HQ_TOTAL] = total;
        out_bytes[0] = total;
    }
}

// ------------------------------------------------------------------------------------------------
template <int S>
static void launch_encode_s(const Geom& g, const void* payload, const Ws& w, uint64_t epoch, uint8_t* out,
                            uint64_t capacity, uint32_t bpt, hipStream_t s) {
    dim3 grid(g.T * bpt), block(256);
    size_t sm = (size_t)g.K * 2;
    const bool f16 = g.dtype == DLC_F16;
#define DLC_ENC(F, V)                                                                                              \
    hipLaunchKernelGGL((k_encode<S, F, V>), grid, block, sm, s, payload, g, w.qp, w.enc, w.group_outliers,            \
                       w.group_out_base, w.layout,                                                                   \
                       w.ctrl, w.state, epoch, out, capacity, bpt, w.word_start, w.word_end)
    if (f16) { if (g.vec) DLC_ENC(true, true); else DLC_ENC(true, false); }
    else { if (g.vec) DLC_ENC(false, true); else DLC_ENC(false, false); }
#undef DLC_ENC
}

hipError_t launch_compress(const Geom& g, const void* payload, uint8_t* out, uint64_t capacity, uint64_t* out_bytes,
                           const Ws& w, uint64_t epoch, int pl, void* prof, hipStream_t s) {
    const bool f16 = g.dtype == DLC_F16;
    // clear histograms, escape totals, ticket and abort flag
    {
        const size_t n16 = (size_t)(w.zero_end - w.zero_begin) / 16;
        if (prof_on(pl, P_ZERO)) prof_begin(prof, P_ZERO, s);
        hipLaunchKernelGGL(k_zero, dim3((unsigned)std::min<size_t>((n16 + 255) / 256, 1024)), dim3(256), 0, s,
                           reinterpret_cast<uint4*>(w.zero_begin), n16);
        if (prof_on(pl, P_ZERO)) prof_end(prof, P_ZERO, s);
    }
    // histogram: up to 8 copies of each bin, 32 KiB of LDS at most
#ifndef DLC_EXP_HIST_CLOG2
#define DLC_EXP_HIST_CLOG2 3
#endif
    uint32_t clog2 = DLC_EXP_HIST_CLOG2;
    while (clog2 > 0 && ((size_t)g.K << clog2) * 4 > 32768) --clog2;
    const uint32_t waves_per_table = g.G;
    uint32_t bpt_h = (waves_per_table + 3) / 4;
    {
        // cap the grid at a few work-groups per CU; a work-group then loops over groups of its table
#ifndef DLC_EXP_HIST_BLOCKS
#define DLC_EXP_HIST_BLOCKS (256 * 8)
#endif
        const uint32_t max_blocks = DLC_EXP_HIST_BLOCKS;
        const uint32_t cap = std::max<uint32_t>(1, max_blocks / g.T);
        bpt_h = std::min(bpt_h, cap);
        size_t sm = ((size_t)g.K << clog2) * 4 + kW * 4;  // + one scratch bin per lane
        dim3 grid(g.T * bpt_h), block(256);
        if (prof_on(pl, P_HIST)) prof_begin(prof, P_HIST, s);
#define DLC_HIST(F, V)                                                                                          \
    hipLaunchKernelGGL((k_hist<F, V>), grid, block, sm, s, payload, g, w.qp, w.hist, w.group_outliers,           \
                       w.table_outliers, bpt_h, clog2)
        if (f16) { if (g.vec) DLC_HIST(true, true); else DLC_HIST(true, false); }
        else { if (g.vec) DLC_HIST(false, true); else DLC_HIST(false, false); }
#undef DLC_HIST
        if (prof_on(pl, P_HIST)) prof_end(prof, P_HIST, s);
    }
    if (prof_on(pl, P_CODEBOOK)) prof_begin(prof, P_CODEBOOK, s);
    hipLaunchKernelGGL(k_codebook, dim3(g.T), dim3(256), codebook_smem(g.K), s, g, w.hist, w.table_outliers, w.enc,
                       w.lens, w.tmeta);
    if (prof_on(pl, P_CODEBOOK)) prof_end(prof, P_CODEBOOK, s);
    if (prof_on(pl, P_LAYOUT)) prof_begin(prof, P_LAYOUT, s);
    hipLaunchKernelGGL(k_layout, dim3(1), dim3(1024), 0, s, g, w.tmeta, w.group_outliers, w.group_out_base, w.lens, w.qp,
                       out, capacity, w.ctrl, w.layout);
    if (prof_on(pl, P_LAYOUT)) prof_end(prof, P_LAYOUT, s);
    {
        const uint32_t bpt = (g.G + 3) / 4;
        if (prof_on(pl, P_ENCODE)) prof_begin(prof, P_ENCODE, s);
        switch (g.S) {
            case 64: launch_encode_s<64>(g, payload, w, epoch, out, capacity, bpt, s); break;
            case 128: launch_encode_s<128>(g, payload, w, epoch, out, capacity, bpt, s); break;
            default: launch_encode_s<256>(g, payload, w, epoch, out, capacity, bpt, s); break;
        }
        if (prof_on(pl, P_ENCODE)) prof_end(prof, P_ENCODE, s);
    }
    if (prof_on(pl, P_FINALIZE)) prof_begin(prof, P_FINALIZE, s);
    hipLaunchKernelGGL(k_finalize, dim3(1), dim3(256), 0, s, g, w.tmeta, w.layout, w.ctrl, w.word_start, w.word_end, out,
                       out_bytes);
    if (prof_on(pl, P_FINALIZE)) prof_end(prof, P_FINALIZE, s);
    return hipGetLastError();
}

hipError_t compress_set_attributes() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k_codebook), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)codebook_smem(4096));
}

}  // namespace dlc
