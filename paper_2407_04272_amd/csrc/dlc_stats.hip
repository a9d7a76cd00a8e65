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

// pass 1: one wavefront per row (grid-stride over the rows of a table)
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
    for (uint32_t row = wave_global; row < g.B; row += rows_grid) {
        uint64_t hr = 0, hq = 0;
        for (uint32_t e = lane; e < g.D; e += 64) {
            uint32_t raw;
            const float x = elem_at<F16>(tab, row * g.D + e, raw);
            if (__builtin_fabsf(x) < __builtin_inff()) {
                const uint32_t o = ord_enc(x);
                mn = min(mn, o);
                mx = max(mx, o);
            }
            const uint32_t c = quant_symbol<F16>(x, q, Rf, (int)g.R);
            const uint64_t pos = (uint64_t)(e + 1u) * 0x9E3779B97F4A7C15ull + salt;
            hr += mix64((uint64_t)raw + pos);
            hq += mix64((uint64_t)c + pos);
        }
        hr = mix64(wave_sum64(hr)) | 1ull;  // never 0: 0 marks an empty slot
        hq = mix64(wave_sum64(hq)) | 1ull;
        if (lane < 2) {
            const uint64_t hsh = lane == 0 ? hr : hq;
            const size_t set = (size_t)lane * g.T + t;
            rowhash[set * g.B + row] = hsh;
            uint64_t* kk = keys + set * M;
            uint32_t* oo = owner + set * M;
            uint32_t pos = (uint32_t)(hsh >> 20) & (M - 1u);
            for (uint32_t probe_n = 0; probe_n < M; ++probe_n) {
                const uint64_t prev = atomicCAS(reinterpret_cast<unsigned long long*>(&kk[pos]), 0ull,
                                                (unsigned long long)hsh);
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

// pass 2: a row is distinct iff it owns its slot; every other row must equal the owner
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
    for (uint32_t row = wave_global; row < g.B; row += rows_grid) {
        for (uint32_t set_i = 0; set_i < 2; ++set_i) {
            const size_t set = (size_t)set_i * g.T + t;
            const uint64_t hsh = rowhash[set * g.B + row];
            const uint64_t* kk = keys + set * M;
            uint32_t pos = (uint32_t)(hsh >> 20) & (M - 1u);
            uint32_t own = 0xFFFFFFFFu;
            for (uint32_t probe_n = 0; probe_n < M; ++probe_n) {
                if (kk[pos] == hsh) { own = owner[set * M + pos]; break; }
                pos = (pos + 1u) & (M - 1u);
            }
            if (own == row) {
                if (set_i == 0) ++n_raw; else ++n_quant;
                continue;
            }
            if (own >= g.B) {  // the set was too small or was not filled: an internal error
                if (lane == 0) set_status(ctrl, DLC_ESTATE);
                continue;
            }
            bool differ = false;
            for (uint32_t e = lane; e < g.D; e += 64) {
                uint32_t ra, rb;
                const float xa = elem_at<F16>(tab, row * g.D + e, ra);
                const float xb = elem_at<F16>(tab, own * g.D + e, rb);
                if (set_i == 0) differ |= ra != rb;
                else differ |= quant_symbol<F16>(xa, q, Rf, (int)g.R) != quant_symbol<F16>(xb, q, Rf, (int)g.R);
            }
            if (__ballot(differ) != 0ull && lane == 0) atomicAdd(&ctrl->collide, 1u);
        }
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
    const uint32_t blocks_x = std::min<uint32_t>((g.B + 3) / 4, DLC_STATS_BLOCKS);
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
