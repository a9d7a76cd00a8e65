// Device-side building blocks shared by the compression kernels of libdlc (gfx950 only): the LDS histogram
// layout, the Huffman codebook builder, the look-back scan over groups and the bit-stream writer.
#pragma once
#include "dlc_internal.h"

// phase time stamps for kernel micro-benchmarks; expands to nothing in the library

namespace dlc {

// ------------------------------------------------------------------------------------------------
// The symbol window.  Almost every element of a bell-shaped table falls into a few bins around zero, so the
// streaming kernels work on window indices: index v in [0, 254) stands for symbol win_lo + v, index 254 for an
// escape, index 255 for everything else (a symbol outside the window, a position past the end of the table).
//   - the histogram kernel counts window indices in LDS with kWinCopies copies per row (copy = lane mod
//     kWinCopies, so a wavefront's 64 updates spread over the banks whatever the symbols are) and hands the
//     indices on as one byte per element (the symbol plane); the rare index 255 is counted exactly by symbol, the
//     escapes in row 254
//   - the encode kernel looks window indices up in a 256-entry LDS table and goes back to the element itself
//     only for index 255
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kWinBins = 255;   // index of "see the element itself" (a symbol outside the window, a position past the end)
constexpr uint32_t kWinEsc = 254;    // index of an escape: its code comes from the table like any other, its record from the payload
constexpr uint32_t kWinSkip = 253;   // with row matching: an element of a row that is stored as a reference (no bits)
// window indices that stand for a symbol: [0, win_bins)
__host__ __device__ inline uint32_t win_bins(uint32_t lz) { return lz ? kWinSkip : kWinEsc; }
constexpr uint32_t kWinCopies = 16;
__host__ __device__ inline uint32_t win_lo_of(uint32_t R) { return R > kWinBins / 2u ? R - kWinBins / 2u : 0u; }
// The symbol plane: the window index of every element, one byte each, in element order; a table's part is padded to
// whole groups (and the last unit of a table is always written whole), so that every group has its 64*S bytes.
__host__ __device__ inline size_t plane_stride(const Geom& g) { return (size_t)g.G * kW * g.S; }
// LDS of the histogram kernel in words: window [kWinBins + 1][kWinCopies] | exact counts [K]
__host__ __device__ inline size_t hist_lds_bytes(uint32_t K) { return (((size_t)(kWinBins + 1) * kWinCopies + K) * 4 + 15) & ~size_t(15); }

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
    uint32_t lo, hi, maxlen, codes_done, cl[kLmaxLimit + 2], next[kLmaxLimit + 2];
};

__device__ __forceinline__ uint32_t lane_get(uint32_t v, uint32_t l) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)__builtin_amdgcn_readfirstlane((int)(l & 63u)));
}
__device__ __forceinline__ uint32_t lane_put(uint32_t vec, uint32_t l, uint32_t val, uint32_t lane) {
    return lane == l ? val : vec;
}

// lane read with a wavefront-uniform lane number that the compiler can see is uniform (no broadcast of the number first)
__device__ __forceinline__ uint32_t lane_read(uint32_t v, uint32_t l) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)l);
}

// The whole tree of a table with at most 64 used symbols, built by one wavefront without touching memory:
// lane i holds used symbol i (symbol order) on entry.  Leaves and merged nodes live one per lane; the merge
// loop runs on wavefront-uniform values only (the queue heads sit in scalar registers, lane reads and writes
// move them); depths come from pointer jumping.  Lengths above LM are limited as described above.  Returns the
// code length of the symbol the lane came in with.  2 <= n <= 64.
__device__ __forceinline__ uint32_t wave_huffman_lengths(uint32_t n, uint32_t LM, uint32_t cnt, uint32_t lane) {
    const uint32_t kInf = 0xFFFFFFFFu;
    // position in (count, symbol) order
    uint32_t rank = 0;
    for (uint32_t j = 0; j < n; ++j) {
        const uint32_t cj = lane_read(cnt, j);
        rank += (cj < cnt || (cj == cnt && j < lane)) ? 1u : 0u;
    }
    if (lane >= n) rank = lane;  // idle lanes keep their place
    // the sorted sequence: every lane sends its count to the lane of its rank
    const uint32_t sent = (uint32_t)__builtin_amdgcn_ds_permute((int)(rank << 2), (int)cnt);
    const uint32_t s_cnt = lane < n ? sent : kInf;
    // two-queue merge; a tie between the heads takes the leaf.  l0, l1: the two leaves at the head of the leaf
    // queue; n0, n1: the same for the merged nodes (node k exists from step k + 1 on)
    const uint32_t vw = s_cnt;
    uint32_t vn = kInf, vpl = 0, vpn = 0;
    uint32_t a = 0, bq = 0;
    uint32_t l0 = lane_read(vw, 0), l1 = lane_read(vw, 1), n0 = kInf, n1 = kInf;
    for (uint32_t k = 0; k + 1 < n; ++k) {
        const bool f_leaf = l0 <= n0;
        const uint32_t s1 = f_leaf ? l0 : n0;
        const uint32_t c_l = f_leaf ? l1 : l0, c_n = f_leaf ? n0 : n1;
        const bool s_leaf = c_l <= c_n;
        const uint32_t s2 = s_leaf ? c_l : c_n;
        if (f_leaf) { vpl = lane_put(vpl, a, k, lane); ++a; } else { vpn = lane_put(vpn, bq, k, lane); ++bq; }
        if (s_leaf) { vpl = lane_put(vpl, a, k, lane); ++a; } else { vpn = lane_put(vpn, bq, k, lane); ++bq; }
        vn = lane_put(vn, k, s1 + s2, lane);
        l0 = a < n ? lane_read(vw, a) : kInf;
        l1 = a + 1u < n ? lane_read(vw, a + 1u) : kInf;
        n0 = bq <= k ? lane_read(vn, bq) : kInf;
        n1 = bq + 1u <= k ? lane_read(vn, bq + 1u) : kInf;
    }
    // depth of every merged node (lane k = node k, the root is node n-2)
    const uint32_t root = n - 2u;
    uint32_t p = (lane < root) ? vpn : lane;
    uint32_t d = (lane < root) ? 1u : 0u;
#pragma unroll
    for (int r = 0; r < 6; ++r) {
        const uint32_t dd = __shfl(d, p, 64), pp = __shfl(p, p, 64);
        d += dd;
        p = pp;
    }
    uint32_t len = lane < n ? __shfl(d, vpl, 64) + 1u : 0u;  // of the leaf at sorted position `lane`
    uint32_t m = len;
    for (int o = 32; o > 0; o >>= 1) m = max(m, (uint32_t)__shfl_xor(m, o, 64));
    if (m > LM) {
        // cut to LM, then repair the Kraft sum: a code of length LM pairs up with a code taken from the deepest
        // shorter level, one unit at a time.  Lane L of clv holds the number of codes of length L.
        const uint32_t lc = min(len, LM);
        uint32_t clv = 0;
        uint64_t kraft = 0;  // in units of 2^-LM
        for (uint32_t L = 1; L <= LM; ++L) {
            const uint32_t c = (uint32_t)__popcll(__ballot(lane < n && lc == L));
            clv = lane_put(clv, L, c, lane);
            kraft += (uint64_t)c << (LM - L);
        }
        while (kraft > (1ull << LM) && lane_get(clv, LM) > 0u) {
            const uint64_t shorter = __ballot(clv > 0u && lane >= 1u && lane < LM);
            clv = lane_put(clv, LM, lane_get(clv, LM) - 1u, lane);
            if (shorter) {
                const uint32_t Ld = 63u - (uint32_t)__builtin_clzll(shorter);
                clv = lane_put(clv, Ld, lane_get(clv, Ld) - 1u, lane);
                clv = lane_put(clv, Ld + 1u, lane_get(clv, Ld + 1u) + 2u, lane);
            }
            kraft -= 1;
        }
        // lengths are handed out most frequent leaf first (the leaves are sorted by rising count)
        const uint32_t back = n - 1u - lane;
        uint32_t acc = 0, nl = 1;
        for (uint32_t L = 1; L < LM; ++L) {
            acc += lane_get(clv, L);  // leaves with a length of at most L
            nl += (back >= acc) ? 1u : 0u;
        }
        len = lane < n ? nl : 0u;
    }
    // back to symbol order: the lane that came in with a symbol reads the length at that symbol's sorted position
    return lane < n ? __shfl(len, rank, 64) : 0u;
}

// The codebook of a table with at most 64 used symbols (the rule), by ONE wavefront: same inputs and outputs as
// codebook_build below, which takes every other table.  The wavefront reads the histogram 64 symbols at a time,
// gathers the used symbols into its lanes through `wsm` (LDS of this wavefront: 64 keys, then K entries of 16
// bits), builds the tree in registers, and writes the K entries of the table and the code lengths.  Returns false,
// with the histogram untouched, when the table has more than 64 used symbols.
//   wsm: 512 + 2 * K bytes, 8-byte aligned.
__host__ __device__ constexpr size_t codebook_wave_smem(uint32_t K) { return 512 + 2 * (size_t)K; }
__device__ __forceinline__ bool codebook_build_wave(const Geom& g, uint32_t* hist_t, uint32_t* hist_view_t, uint16_t* enc_t,
                                                    uint8_t* lens_t, TMeta* tmeta_t, unsigned char* wsm, uint32_t lane,
                                                    uint32_t carry) {
    const uint32_t K = g.K;  // (a multiple of 64: twice a power of two of at least 8)
    uint64_t* key = reinterpret_cast<uint64_t*>(wsm);            // [64] count << 16 | symbol of the used symbols, symbol order
    uint16_t* ent = reinterpret_cast<uint16_t*>(wsm + 512);      // [K] len << 12 | codeword
    const uint64_t below = (1ull << lane) - 1ull;
    uint32_t n_used = 0, n_escape = 0;
    for (uint32_t kb = 0; kb < K; kb += 16u * 64u) {  // sixteen loads of 64 symbols in flight together
        // the counts were added by device-scope atomics of other work-groups, possibly on other dies
        uint32_t hv[16];
#pragma unroll
        for (uint32_t i = 0; i < 16; ++i)
            hv[i] = kb + i * 64u < K ? __hip_atomic_load(&hist_t[kb + i * 64u + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
#pragma unroll
        for (uint32_t i = 0; i < 16; ++i) {
            const uint32_t k = kb + i * 64u + lane;
            if (kb + i * 64u >= K) continue;  // uniform
            const uint32_t h = hv[i];
            // a codebook that is carried to the next call always has a code for the escape symbol
            const uint32_t c = h + ((carry != 0u && k == 0u) ? 1u : 0u);
            if (hist_t != hist_view_t) hist_view_t[k] = h;  // (the copy itself can be the source: it is left as it is)
            if (kb + i == 0u) n_escape = (uint32_t)__builtin_amdgcn_readfirstlane((int)c);
            ent[k] = 0;
            const uint64_t m = __ballot(c != 0u);
            const uint32_t at = n_used + (uint32_t)__popcll(m & below);
            if (c != 0u && at < 64u) key[at] = ((uint64_t)c << 16) | k;
            n_used += (uint32_t)__popcll(m);
        }
    }
    if (n_used > 64u) return false;  // uniform
    if (hist_t != hist_view_t)
        for (uint32_t k0 = 0; k0 < K; k0 += 64)
            __hip_atomic_store(&hist_t[k0 + lane], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_wave_barrier();
    const uint64_t kv = lane < n_used ? key[lane] : ~0ull;  // lane i: the i-th used symbol
    const uint32_t sym = (uint32_t)(kv & 0xFFFFu);
    if (n_used >= 2u) {
        const uint32_t len = wave_huffman_lengths(n_used, g.LMAX, (uint32_t)(kv >> 16), lane);
        // canonical codewords: first code of each length, then the rank among the symbols of that length (the lanes
        // are in symbol order)
        uint32_t code = 0, mine_code = 0;
        for (uint32_t L = 1; L <= g.LMAX; ++L) {
            code <<= 1;
            const uint64_t same = __ballot(len == L);
            mine_code = (len == L) ? code + (uint32_t)__popcll(same & below) : mine_code;
            code += (uint32_t)__popcll(same);
        }
        if (lane < n_used) ent[sym] = (uint16_t)((len << 12) | mine_code);
    }
    __builtin_amdgcn_wave_barrier();
    for (uint32_t k0 = 0; k0 < K; k0 += 64) {
        const uint32_t e = ent[k0 + lane];
        __hip_atomic_store(&enc_t[k0 + lane], (uint16_t)e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lens_t[k0 + lane] = (uint8_t)(e >> 12);
    }
    if (lane == 0) {
        TMeta m;
        m.n_used = n_used;
        m.sym_lo = n_used ? (uint32_t)(key[0] & 0xFFFFu) : 0u;
        m.sym_hi = n_used ? (uint32_t)(key[n_used - 1u] & 0xFFFFu) : 0u;
        m.n_outliers = n_escape;  // symbol 0 = escape
        *tmeta_t = m;
    }
    return true;
}

// A work-group of four wavefronts builds the codebooks of the tables [t0, t0 + 4): a wavefront each where the table
// has at most 64 used symbols, the whole work-group one after the other for the rest.
//   smem: codebook_smem(K) bytes, 16-byte aligned (the wavefronts' areas lie inside it).
// hist_t is read, copied to hist_view_t (inspection) and cleared, so that the next call starts from zero counts.
// enc_t is written with device-scope stores: other work-groups of a running kernel may read it once they have
// seen the caller's completion flag.
__device__ __forceinline__ void codebook_build(const Geom& g, uint32_t* hist_t, uint32_t* hist_view_t, uint16_t* enc_t,
                                               uint8_t* lens_t, TMeta* tmeta_t, unsigned char* smem, CodebookShared& sh,
                                               uint32_t tid, uint32_t carry = 0) {
    const uint32_t K = g.K;
    uint64_t* key = reinterpret_cast<uint64_t*>(smem);        // [K] sort keys: count << 16 | symbol
    uint32_t* cnt = reinterpret_cast<uint32_t*>(key + K);      // [K] counts
    uint32_t* nodew = cnt + K;                                 // [K] merged-node weights, later codewords
    uint16_t* parent_leaf = reinterpret_cast<uint16_t*>(nodew + K);  // [K] parent of a leaf, later its length
    uint16_t* parent_node = parent_leaf + K;                   // [K]
    uint16_t* depth_node = parent_node + K;                    // [K]
    uint16_t* len_s = depth_node + K;                          // [K] code length per symbol
    uint32_t* scratch = reinterpret_cast<uint32_t*>(len_s + K);  // [64]
    const uint32_t lane = tid & 63u, wave = tid >> 6;

    // each thread owns `per` consecutive symbols
    const uint32_t per = (K + 255) / 256;
    const uint32_t k0 = tid * per, k1 = min(K, k0 + per);
    uint32_t mine = 0;
    // the counts were added by device-scope atomics of other work-groups, possibly on other dies; a thread's loads
    // go out together (at most 16: an alphabet of 4096 symbols)
    uint32_t hv[16];
#pragma unroll
    for (uint32_t i = 0; i < 16; ++i)
        hv[i] = k0 + i < k1 ? __hip_atomic_load(&hist_t[k0 + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
#pragma unroll
    for (uint32_t i = 0; i < 16; ++i) {
        const uint32_t k = k0 + i;
        if (k >= k1) break;
        const uint32_t h = hv[i];
        // a codebook that is carried to the next call always has a code for the escape symbol
        cnt[k] = h + ((carry != 0u && k == 0u) ? 1u : 0u);
        if (hist_t != hist_view_t) {  // (the copy itself can be the source: it is left as it is)
            hist_view_t[k] = h;
            __hip_atomic_store(&hist_t[k], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        len_s[k] = 0;
        mine += cnt[k] != 0;
    }
    if (tid == 0) { sh.maxlen = 0; sh.codes_done = 0; }
    if (tid < kLmaxLimit + 2) sh.cl[tid] = 0;
    // compaction offsets of the used symbols (symbol order); the barriers inside also publish cnt[]
    uint32_t n_used;
    const uint32_t my_off = block_excl_scan<4>(mine, scratch, tid, &n_used);
    {
        uint32_t o = my_off;
        for (uint32_t k = k0; k < k1; ++k)
            if (cnt[k]) key[o++] = ((uint64_t)cnt[k] << 16) | k;
    }
    __syncthreads();
    // first and last used symbol: the ends of the compacted list
    const uint32_t sym_lo = n_used ? (uint32_t)(key[0] & 0xFFFFu) : 0u;
    const uint32_t sym_hi = n_used ? (uint32_t)(key[n_used - 1] & 0xFFFFu) : 0u;

    if (n_used >= 2 && n_used <= 64) {
        if (wave == 0) {
            const uint64_t kv = lane < n_used ? key[lane] : ~0ull;  // lane i: the i-th used symbol
            const uint32_t sym = (uint32_t)(kv & 0xFFFFu);
            const uint32_t len = wave_huffman_lengths(n_used, g.LMAX, (uint32_t)(kv >> 16), lane);
            // canonical codewords: first code of each length, then the rank among the symbols of that length (the
            // lanes are in symbol order)
            const uint64_t below = (1ull << lane) - 1ull;
            uint32_t code = 0, mine_code = 0;
            for (uint32_t L = 1; L <= g.LMAX; ++L) {
                code <<= 1;
                const uint64_t same = __ballot(len == L);
                mine_code = (len == L) ? code + (uint32_t)__popcll(same & below) : mine_code;
                code += (uint32_t)__popcll(same);
            }
            if (lane < n_used) { len_s[sym] = (uint16_t)len; nodew[sym] = mine_code; }
            if (lane == 0) sh.codes_done = 1;
        }
        __syncthreads();
    } else if (n_used > 64) {
        const uint32_t n_escape = cnt[0];  // (cnt[] is scratch from here on:
        __syncthreads();                   //  once every thread has read this)
        if (n_used <= 256) {
            // rank sort, a thread per key: the keys are distinct (the symbol is part of them), so a key's place is
            // the number of smaller keys; every thread reads the same key at a time (an LDS broadcast)
            uint64_t* tmp = reinterpret_cast<uint64_t*>(cnt);  // cnt[] and nodew[] together: K words of 64 bits
            uint64_t mykey = 0;
            uint32_t rank = 0;
            if (tid < n_used) {
                mykey = key[tid];
                for (uint32_t j = 0; j < n_used; ++j) rank += key[j] < mykey ? 1u : 0u;
                tmp[rank] = mykey;
            }
            __syncthreads();
            if (tid < n_used) key[tid] = tmp[tid];
            __syncthreads();
        } else {
            uint32_t P = 2;
            while (P < n_used) P <<= 1;
            for (uint32_t i = n_used + tid; i < P; i += 256) key[i] = ~0ull;  // pad to a power of two
            __syncthreads();
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
        }
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
        }
        __syncthreads();
        {
            // depth of every merged node by pointer jumping (the root, node n - 2, points at itself at distance 0):
            // after round r a node knows its 2^r-th ancestor and the distance to it.  Two buffers of packed
            // (distance << 16 | ancestor) words, in cnt[] and nodew[], which are both free here.
            const uint32_t root = n_used - 2u;
            uint32_t* cur = cnt;
            uint32_t* nxt = nodew;
            for (uint32_t k = tid; k + 1 < n_used; k += 256) cur[k] = k == root ? root : ((1u << 16) | parent_node[k]);
            __syncthreads();
            for (uint32_t span = 1; span < n_used; span <<= 1) {  // uniform trip count
                for (uint32_t k = tid; k + 1 < n_used; k += 256) {
                    const uint32_t me = cur[k], up = cur[me & 0xFFFFu];
                    nxt[k] = ((me >> 16) + (up >> 16)) << 16 | (up & 0xFFFFu);
                }
                __syncthreads();
                uint32_t* sw = cur; cur = nxt; nxt = sw;
            }
            for (uint32_t k = tid; k + 1 < n_used; k += 256) depth_node[k] = (uint16_t)(cur[k] >> 16);
            __syncthreads();
            if (tid == 0) cnt[0] = n_escape;  // read again at the end (nothing below writes cnt[])
        }
        // leaf depths; parent_leaf[] is reused to hold the depth of leaf i (sorted order)
        uint32_t local_max = 0;
        for (uint32_t i = tid; i < n_used; i += 256) {
            const uint32_t d = depth_node[parent_leaf[i]] + 1u;
            parent_leaf[i] = (uint16_t)d;
            local_max = max(local_max, d);
        }
        if (local_max) atomicMax(&sh.maxlen, local_max);
        __syncthreads();
    }
    if (n_used >= 2) {
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
        if (!sh.codes_done) {  // uniform
            for (uint32_t i = tid; i < n_used; i += 256) len_s[(uint32_t)(key[i] & 0xFFFFu)] = parent_leaf[i];
            __syncthreads();
            // codewords
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
            }
            __syncthreads();
            // a symbol's codeword: the first code of its length plus the number of smaller symbols of that length
            for (uint32_t k = sym_lo + tid; k <= sym_hi; k += 256) {
                const uint32_t L = len_s[k];
                if (L) {
                    uint32_t r = 0;
                    for (uint32_t j = sym_lo; j < k; ++j) r += len_s[j] == L ? 1u : 0u;
                    nodew[k] = sh.next[L] + r;
                }
            }
            __syncthreads();
        }
    }
    for (uint32_t k = k0; k < k1; ++k) {
        uint32_t L = len_s[k];
        __hip_atomic_store(&enc_t[k], (uint16_t)(L ? ((L << 12) | nodew[k]) : 0u), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        lens_t[k] = (uint8_t)L;
    }
    if (tid == 0) {
        TMeta m;
        // an empty histogram cannot come out of the histogram step (every table has an element); should it
        // happen anyway, the symbol range is still a valid one for the kernels that size things from it
        m.n_used = n_used; m.sym_lo = sym_lo; m.sym_hi = sym_hi; m.n_outliers = cnt[0];  // symbol 0 = escape
        *tmeta_t = m;
    }
    __syncthreads();
}

__device__ __forceinline__ void codebook_build_four(const Geom& g, uint32_t t0, uint32_t* hist, uint32_t* hist_view, uint16_t* enc,
                                                    uint8_t* lens, TMeta* tmeta, unsigned char* smem, CodebookShared& sh,
                                                    uint32_t* slow, uint32_t tid, uint32_t carry) {
    static_assert(4 * (512 + 2 * 4096) <= 4096 * 24 + 256, "the wavefronts' areas must fit the work-group's");
    const uint32_t lane = tid & 63u, wave = tid >> 6, t = t0 + wave;
    if (t < g.T) {  // uniform over the wavefront
        const bool done = codebook_build_wave(g, hist + (size_t)t * g.K, hist_view + (size_t)t * g.K, enc + (size_t)t * g.K,
                                              lens + (size_t)t * g.K, tmeta + t, smem + wave * codebook_wave_smem(g.K), lane, carry);
        if (lane == 0) slow[wave] = done ? 0u : 1u;
    } else if (lane == 0) {
        slow[wave] = 0u;
    }
    __syncthreads();
    for (uint32_t w = 0; w < 4; ++w) {
        if (slow[w] == 0u) continue;  // uniform over the work-group
        const uint32_t ts = t0 + w;
        codebook_build(g, hist + (size_t)ts * g.K, hist_view + (size_t)ts * g.K, enc + (size_t)ts * g.K, lens + (size_t)ts * g.K,
                       tmeta + ts, smem, sh, tid, carry);
    }
}

// ------------------------------------------------------------------------------------------------
// offsets of the output: single-pass look-back scan
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kFlagAgg = 1, kFlagPrefix = 2;
constexpr uint32_t kSpinLimit = 1u << 22;

// Exclusive prefix of `total` over the work-groups before `wg`: single-pass look-back over one record per
// work-group, 256 records per step (four per lane).  The chain of "wait for a predecessor's prefix" steps across
// the work-groups that run at the same time is what bounds a streaming kernel that places its output by such a
// scan, so the records are few and the steps wide.  Publishes this work-group's records.  Called by one whole
// wavefront.
// dom0: the first work-group of this work-group's scan domain (a destination's container: offsets start at 0 there).
__device__ __forceinline__ uint32_t wg_scan(uint64_t* state, uint64_t epoch, uint32_t wg, uint32_t total, uint32_t lane,
                                            Ctrl* ctrl, bool* dead, uint32_t dom0 = 0) {
    const uint64_t tag = epoch << 34;
    if (lane == 0)
        __hip_atomic_store(&state[wg], tag | ((uint64_t)(wg == dom0 ? kFlagPrefix : kFlagAgg) << 32) | total,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t excl = 0;
    if (wg > dom0) {
        int64_t pos = (int64_t)wg - 1;  // nearest record not yet added
        uint32_t spins = 0;
        for (;;) {
            // this lane's four records, nearest first; before the first work-group: an empty prefix
            uint32_t sum = 0;       // values up to and including the lane's first prefix record (or all four)
            bool has_p = false;     // there is a prefix record among them
            bool hole = false;      // an unpublished record comes before it
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int64_t my = pos - (int64_t)(lane * 4u + (uint32_t)k);
                const uint64_t sv = my >= (int64_t)dom0 ? __hip_atomic_load(&state[my], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                                        : (tag | ((uint64_t)kFlagPrefix << 32));
                const uint32_t flag = (sv >> 34) == epoch ? (uint32_t)(sv >> 32) & 3u : 0u;
                if (!has_p) {
                    hole = hole || flag == 0u;
                    sum += flag != 0u ? (uint32_t)sv : 0u;
                    has_p = flag == kFlagPrefix;
                }
            }
            const uint64_t pm = __ballot(has_p);
            const uint32_t first = pm ? (uint32_t)__ffsll((unsigned long long)pm) - 1u : 64u;  // lane of the nearest prefix
            if (__ballot(hole && lane <= first) != 0ull) {  // something nearer than that prefix is not published yet
                if (++spins > kSpinLimit) {  // never expected; the bound only guarantees termination
                    if (lane == 0) { set_status(ctrl, DLC_ESTATE); atomicOr(&ctrl->abort, kAbortInternal); }
                    *dead = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
                continue;
            }
            excl += wave_sum(lane <= first ? sum : 0u);
            if (pm) break;
            pos -= 256;
        }
        if (lane == 0)
            __hip_atomic_store(&state[wg], tag | ((uint64_t)kFlagPrefix << 32) | (uint32_t)(excl + total),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return excl;
}

// The same look-back in steps that can be spread through other work: issue() starts the loads of one step,
// consume() uses them.  Between the two the caller does something else, so the latency of the records (they
// live in device-coherent memory, a few hundred nanoseconds away) costs nothing.  The caller has published its
// own aggregate record before the first step (publish_aggregate) and publishes the prefix when done.
struct LookBack {
    int64_t dom0;     // first work-group of the scan domain (records before it count as an empty prefix)
    int64_t pos;      // nearest record not yet added
    uint32_t excl;    // sum so far
    uint32_t spins;
    bool done, failed, pending;
    uint64_t sv[4];
};

__device__ __forceinline__ void lb_publish_aggregate(uint64_t* state, uint64_t epoch, uint32_t wg, uint32_t total, uint32_t lane,
                                                     uint32_t dom0 = 0) {
    if (lane == 0)
        __hip_atomic_store(&state[wg], (epoch << 34) | ((uint64_t)(wg == dom0 ? kFlagPrefix : kFlagAgg) << 32) | total,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void lb_init(LookBack& L, uint32_t wg, uint32_t dom0 = 0) {
    L.dom0 = (int64_t)dom0;
    L.pos = (int64_t)wg - 1;
    L.excl = 0;
    L.spins = 0;
    L.done = wg == dom0;
    L.failed = false;
    L.pending = false;
}
__device__ __forceinline__ void lb_issue(LookBack& L, const uint64_t* state, uint64_t epoch, uint32_t lane) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t my = L.pos - (int64_t)(lane * 4u + (uint32_t)k);
        L.sv[k] = my >= L.dom0 ? __hip_atomic_load(&state[my], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                               : ((epoch << 34) | ((uint64_t)kFlagPrefix << 32));  // before the domain's first work-group: an empty prefix
    }
    L.pending = true;
}
// true if the step made progress (false: a record nearer than the nearest prefix is not published yet)
__device__ __forceinline__ bool lb_consume(LookBack& L, uint64_t epoch, uint32_t lane) {
    uint32_t sum = 0;    // values up to and including the lane's first prefix record (or all four)
    bool has_p = false;  // there is a prefix record among them
    bool hole = false;   // an unpublished record comes before it
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint64_t sv = L.sv[k];
        const uint32_t flag = (sv >> 34) == epoch ? (uint32_t)(sv >> 32) & 3u : 0u;
        if (!has_p) {
            hole = hole || flag == 0u;
            sum += flag != 0u ? (uint32_t)sv : 0u;
            has_p = flag == kFlagPrefix;
        }
    }
    L.pending = false;
    const uint64_t pm = __ballot(has_p);
    const uint32_t first = pm ? (uint32_t)__ffsll((unsigned long long)pm) - 1u : 64u;  // lane of the nearest prefix
    if (__ballot(hole && lane <= first) != 0ull) return false;
    L.excl += wave_sum(lane <= first ? sum : 0u);
    if (pm) L.done = true;
    else L.pos -= 256;
    return true;
}
// runs the remaining steps to the end (bounded) and publishes the prefix record
__device__ __forceinline__ void lb_finish(LookBack& L, uint64_t* state, uint64_t epoch, uint32_t wg, uint32_t total, uint32_t lane,
                                          Ctrl* ctrl) {
    while (!L.done && !L.failed) {
        if (!L.pending) lb_issue(L, state, epoch, lane);
        if (!lb_consume(L, epoch, lane)) {
            if (++L.spins > kSpinLimit) {  // never expected; the bound only guarantees termination
                if (lane == 0) { set_status(ctrl, DLC_ESTATE); atomicOr(&ctrl->abort, kAbortInternal); }
                L.failed = true;
            } else {
                __builtin_amdgcn_s_sleep(1);
            }
        }
    }
    if ((int64_t)wg > L.dom0 && !L.failed && lane == 0)
        __hip_atomic_store(&state[wg], (epoch << 34) | ((uint64_t)kFlagPrefix << 32) | (uint32_t)(L.excl + total),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// escape records of one group, in increasing element index, behind its chunk words, for a group with more escapes
// than the encode kernel remembers on the way: a rolled loop over the group's plane words (index 254 marks an
// escape; an element of a row that is stored as a reference has index 253 and no record) and, for the raw bits,
// over its elements
template <int S, bool F16, bool VEC>
__device__ __forceinline__ void emit_escapes(uint32_t* rec, uint32_t lane, const uint8_t* gbase, const uint32_t* plane_g,
                                             uint32_t gstart, uint32_t rem) {
    uint32_t opos = 0;
    for (uint32_t j = 0; j < (uint32_t)S / kV; ++j) {
        const uint32_t off = lane * kV + j * (kW * kV);
        float x[4];
        uint32_t raw[4];
        const uint32_t valid = load4<F16, VEC>(gbase, off, rem, x, raw);
        const uint32_t m = plane_g[j * kW + lane];
        uint32_t esc = 0;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            esc |= (((valid >> v) & 1u) && ((m >> (8 * v)) & 0xFFu) == kWinEsc) ? (1u << v) : 0u;
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

}  // namespace dlc
