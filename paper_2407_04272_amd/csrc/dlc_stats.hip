// Statistics reduction for gfx950: per-table value range and exact distinct-row counts of the raw rows
// and of the rows quantised at a probe bound (the two counts of the Homogenization Index, Eq. 1).
//
// Distinct rows are counted with a per-table open-addressing set keyed by a 64-bit row hash.  The row
// with the smallest index that reached a slot owns it; in a second pass every other row that maps to the
// slot is compared with the owner element by element, so a hash collision between different rows is
// detected (the host then repeats the reduction with another hash salt) and the counts are exact.
#include <algorithm>

#include "dlc_internal.h"

#ifndef DLC_STATS_BLOCKS
#define DLC_STATS_BLOCKS 32
#endif

namespace dlc {

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ uint64_t wave_sum64(uint64_t v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// float <-> unsigned with the same ordering
__device__ __forceinline__ uint32_t ord_enc(float f) {
    uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

template <bool F16>
__device__ __forceinline__ float elem_at(const uint8_t* tab, uint32_t i, uint32_t& raw) {
    if constexpr (F16) {
        raw = reinterpret_cast<const uint16_t*>(tab)[i];
        return __half2float(__ushort_as_half((unsigned short)raw));
    } else {
        raw = reinterpret_cast<const uint32_t*>(tab)[i];
        return __uint_as_float(raw);
    }
}

constexpr uint32_t kRowsPer = 4;  // rows a wavefront works on at a time: their loads and their set operations overlap

// pass 1: a wavefront takes kRowsPer rows at a time (grid-stride over the rows of a table); all lanes hash the
// rows' elements, then lane 2k+s puts row k into set s (0: raw rows, 1: quantised rows)
template <bool F16>
__global__ __launch_bounds__(256) void k_stats_hash(const void* payload, Geom g, const QParam* probe, uint32_t M,
                                                    uint32_t salt, uint64_t* keys, uint32_t* owner, uint64_t* rowhash,
                                                    uint32_t* minmax, uint32_t rows_grid) {
    const uint32_t t = blockIdx.y;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
    const QParam q = probe[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    uint32_t mn = 0xFFFFFFFFu, mx = 0u;
    for (uint32_t row0 = wave_global * kRowsPer; row0 < g.B; row0 += rows_grid * kRowsPer) {
        uint64_t hr[kRowsPer], hq[kRowsPer];
#pragma unroll
        for (uint32_t k = 0; k < kRowsPer; ++k) { hr[k] = 0; hq[k] = 0; }
        for (uint32_t e = lane; e < g.D; e += 64) {
            uint32_t raw[kRowsPer];
            float x[kRowsPer];
#pragma unroll
            for (uint32_t k = 0; k < kRowsPer; ++k)  // a row past the end reads the last row instead; it is not used
                x[k] = elem_at<F16>(tab, min(row0 + k, g.B - 1u) * g.D + e, raw[k]);
            // row hash = sum over the elements of value * m(position), m odd and different for every position and for
            // the two sets (a multilinear hash: rows that differ in one element never collide, others with
            // probability about 2^-63; integer multiplies are the expensive instructions here, and this needs three
            // 32-bit ones per element where a full 64-bit mix of every element needed sixteen)
            const uint64_t pos = (uint64_t)(e + 1u) * 0x9E3779B97F4A7C15ull + salt;
            const uint64_t m_raw = mix64(pos) | 1ull, m_q = mix64(pos ^ 0x5555555555555555ull) | 1ull;
#pragma unroll
            for (uint32_t k = 0; k < kRowsPer; ++k) {
                if (row0 + k < g.B && __builtin_fabsf(x[k]) < __builtin_inff()) {
                    const uint32_t o = ord_enc(x[k]);
                    mn = min(mn, o);
                    mx = max(mx, o);
                }
                const uint32_t c = quant_symbol<F16>(x[k], q, Rf, (int)g.R);
                hr[k] += (uint64_t)raw[k] * m_raw;
                hq[k] += (uint64_t)c * m_q;
            }
        }
        uint64_t hsh = 0;
#pragma unroll
        for (uint32_t k = 0; k < kRowsPer; ++k) {
            const uint64_t a = mix64(wave_sum64(hr[k])) | 1ull;  // never 0: 0 marks an empty slot
            const uint64_t b = mix64(wave_sum64(hq[k])) | 1ull;
            if ((lane >> 1) == k) hsh = (lane & 1u) ? b : a;
        }
        const uint32_t row = row0 + (lane >> 1);
        if (lane < 2 * kRowsPer && row < g.B) {
            const size_t set = (size_t)(lane & 1u) * g.T + t;
            rowhash[set * g.B + row] = hsh;
            uint64_t* kk = keys + set * M;
            uint32_t* oo = owner + set * M;
            uint32_t pos = (uint32_t)(hsh >> 20) & (M - 1u);
            for (uint32_t probe_n = 0; probe_n < M; ++probe_n) {
                const uint64_t prev = atomicCAS(reinterpret_cast<unsigned long long*>(&kk[pos]), 0ull, (unsigned long long)hsh);
                if (prev == 0ull || prev == hsh) {
                    atomicMin(&oo[pos], row);
                    break;
                }
                pos = (pos + 1u) & (M - 1u);
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        mn = min(mn, (uint32_t)__shfl_xor(mn, o, 64));
        mx = max(mx, (uint32_t)__shfl_xor(mx, o, 64));
    }
    if (lane == 0) {
        atomicMin(&minmax[2 * t], mn);
        atomicMax(&minmax[2 * t + 1], mx);
    }
}

// pass 2: a row is distinct iff it owns its slot; every other row must equal the owner.  Lane 2k+s looks row k up
// in set s; the comparisons of all rows that need one are then done together (their loads overlap).
template <bool F16>
__global__ __launch_bounds__(256) void k_stats_verify(const void* payload, Geom g, const QParam* probe, uint32_t M,
                                                      const uint64_t* keys, const uint32_t* owner,
                                                      const uint64_t* rowhash, uint32_t* unique, Ctrl* ctrl,
                                                      uint32_t rows_grid) {
    const uint32_t t = blockIdx.y;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
    const QParam q = probe[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    uint32_t n_raw = 0, n_quant = 0;
    for (uint32_t row0 = wave_global * kRowsPer; row0 < g.B; row0 += rows_grid * kRowsPer) {
        // look-ups
        uint32_t own = 0xFFFFFFFFu;
        {
            const uint32_t row = row0 + (lane >> 1);
            if (lane < 2 * kRowsPer && row < g.B) {
                const size_t set = (size_t)(lane & 1u) * g.T + t;
                const uint64_t hsh = rowhash[set * g.B + row];
                const uint64_t* kk = keys + set * M;
                uint32_t pos = (uint32_t)(hsh >> 20) & (M - 1u);
                for (uint32_t probe_n = 0; probe_n < M; ++probe_n) {
                    if (kk[pos] == hsh) { own = owner[set * M + pos]; break; }
                    pos = (pos + 1u) & (M - 1u);
                }
            }
        }
        uint32_t ownk[2 * kRowsPer];
        bool need[2 * kRowsPer];
#pragma unroll
        for (uint32_t c = 0; c < 2 * kRowsPer; ++c) {
            ownk[c] = __shfl(own, c, 64);
            const uint32_t row = row0 + (c >> 1);
            need[c] = false;
            if (row < g.B) {
                if (ownk[c] == row) {
                    if (c & 1u) ++n_quant; else ++n_raw;
                } else if (ownk[c] >= g.B) {  // the set was too small or was not filled: an internal error
                    if (lane == 0) set_status(ctrl, DLC_ESTATE);
                } else {
                    need[c] = true;
                }
            }
        }
        // comparisons (uniform conditions: every lane holds the same ownk[] and need[])
        bool differ = false;
        for (uint32_t e = lane; e < g.D; e += 64) {
#pragma unroll
            for (uint32_t c = 0; c < 2 * kRowsPer; ++c) {
                if (!need[c]) continue;
                uint32_t ra, rb;
                const float xa = elem_at<F16>(tab, (row0 + (c >> 1)) * g.D + e, ra);
                const float xb = elem_at<F16>(tab, ownk[c] * g.D + e, rb);
                if (c & 1u) differ |= quant_symbol<F16>(xa, q, Rf, (int)g.R) != quant_symbol<F16>(xb, q, Rf, (int)g.R);
                else differ |= ra != rb;
            }
        }
        if (__ballot(differ) != 0ull && lane == 0) atomicAdd(&ctrl->collide, 1u);
    }
    if (lane == 0) {
        if (n_raw) atomicAdd(&unique[2 * t], n_raw);
        if (n_quant) atomicAdd(&unique[2 * t + 1], n_quant);
    }
}

hipError_t launch_stats(const Geom& g, const void* payload, const QParam* probe, const Ws& w, uint32_t M, uint32_t salt,
                        hipStream_t s) {
    // few, long-running work-groups per table: every wavefront ends with atomics on its table's two range words and two
    // counters, and a wavefront per row made those same-address atomics the whole cost of the reduction
    const uint32_t blocks_x = std::min<uint32_t>((g.B + 4 * kRowsPer - 1) / (4 * kRowsPer), DLC_STATS_BLOCKS);
    const uint32_t rows_grid = blocks_x * 4;
    dim3 grid(blocks_x, g.T), block(256);
    if (g.dtype == DLC_F16) {
        hipLaunchKernelGGL(k_stats_hash<true>, grid, block, 0, s, payload, g, probe, M, salt, w.keys, w.owner, w.rowhash,
                           w.st_minmax, rows_grid);
        hipLaunchKernelGGL(k_stats_verify<true>, grid, block, 0, s, payload, g, probe, M, w.keys, w.owner, w.rowhash,
                           w.st_unique, w.ctrl, rows_grid);
    } else {
        hipLaunchKernelGGL(k_stats_hash<false>, grid, block, 0, s, payload, g, probe, M, salt, w.keys, w.owner, w.rowhash,
                           w.st_minmax, rows_grid);
        hipLaunchKernelGGL(k_stats_verify<false>, grid, block, 0, s, payload, g, probe, M, w.keys, w.owner, w.rowhash,
                           w.st_unique, w.ctrl, rows_grid);
    }
    return hipGetLastError();
}

}  // namespace dlc
