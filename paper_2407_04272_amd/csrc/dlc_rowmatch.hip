// Row matching for gfx950 (the vector-based LZ step of Section III-D: the fixed pattern is one embedding vector).
// For every row of a table: the first row of the batch with the same content after quantisation (all symbols
// equal and, where a symbol is the escape, the raw bits too).  Rows that have an earlier equal are not coded by
// the kernels that follow; they are stored as references.
//
// Same machinery as the statistics reduction: a per-table open-addressing set keyed by a 64-bit row hash, the
// smallest row index that reached a slot owns it; a second pass compares every other row of the slot with the
// owner element by element.  A row whose hash meets a different row's (about 2^-33 per table and call for 8192
// rows) stays a coded row: the container is valid, one match is lost.
#include <algorithm>

#include "dlc_internal.h"

namespace dlc {

namespace {

__device__ __forceinline__ uint64_t rm_mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ uint64_t rm_wave_sum64(uint64_t v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// what two elements must agree in to count as equal: the symbol, or for an escape the raw bits (bit 32 set)
template <bool F16>
__device__ __forceinline__ uint64_t rm_identity(const uint8_t* tab, uint32_t i, const QParam& q, float Rf, int R) {
    uint32_t raw;
    float x;
    if constexpr (F16) {
        raw = reinterpret_cast<const uint16_t*>(tab)[i];
        x = __half2float(__ushort_as_half((unsigned short)raw));
    } else {
        raw = reinterpret_cast<const uint32_t*>(tab)[i];
        x = __uint_as_float(raw);
    }
    const uint32_t c = quant_symbol<F16>(x, q, Rf, R);
    return c ? (uint64_t)c : ((1ull << 32) | raw);
}

constexpr uint32_t kRmRows = 4;  // rows a wavefront works on at a time

}  // namespace

// empty sets: key 0, owner "nobody"
__global__ __launch_bounds__(256) void k_rm_clear(uint64_t* keys, uint32_t* owner, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        keys[i] = 0ull;
        owner[i] = 0xFFFFFFFFu;
    }
}

// pass 1: hash kRmRows rows at a time per wavefront, lane k puts row k into the table's set
template <bool F16>
__global__ __launch_bounds__(256) void k_rm_hash(const void* payload, Geom g, const QParam* qp, const uint8_t* on, uint32_t M,
                                                 uint64_t* keys, uint32_t* owner, uint64_t* rowhash, uint32_t rows_grid) {
    const uint32_t t = blockIdx.y;
    if (!on[t]) return;  // uniform: the table is coded row by row as it is
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    uint64_t* kk = keys + (size_t)t * M;
    uint32_t* oo = owner + (size_t)t * M;
    for (uint32_t row0 = wave_global * kRmRows; row0 < g.B; row0 += rows_grid * kRmRows) {
        uint64_t h[kRmRows];
#pragma unroll
        for (uint32_t k = 0; k < kRmRows; ++k) h[k] = 0;
        for (uint32_t e = lane; e < g.D; e += 64) {
            // multilinear hash: identity times an odd multiplier that depends on the position
            const uint64_t pos = (uint64_t)(e + 1u) * 0x9E3779B97F4A7C15ull;
            const uint64_t m_lo = rm_mix64(pos) | 1ull, m_hi = rm_mix64(pos ^ 0x5555555555555555ull) | 1ull;
#pragma unroll
            for (uint32_t k = 0; k < kRmRows; ++k) {  // a row past the end reads the last row instead; it is not used
                const uint64_t id = rm_identity<F16>(tab, min(row0 + k, g.B - 1u) * g.D + e, q, Rf, (int)g.R);
                h[k] += (uint64_t)(uint32_t)id * m_lo + ((id >> 32) ? m_hi : 0ull);
            }
        }
        uint64_t hsh = 0;
#pragma unroll
        for (uint32_t k = 0; k < kRmRows; ++k) {
            const uint64_t a = rm_mix64(rm_wave_sum64(h[k])) | 1ull;  // never 0: 0 marks an empty slot
            if (lane == k) hsh = a;
        }
        const uint32_t row = row0 + lane;
        if (lane < kRmRows && row < g.B) {
            rowhash[(size_t)t * g.B + row] = hsh;
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
}

// pass 2: ref[row] = the slot's owner if the two rows are equal element by element, else the row itself
template <bool F16>
__global__ __launch_bounds__(256) void k_rm_owner(const void* payload, Geom g, const QParam* qp, const uint8_t* on, uint32_t M,
                                                  const uint64_t* keys, const uint32_t* owner, const uint64_t* rowhash,
                                                  uint32_t* ref, uint32_t rows_grid) {
    const uint32_t t = blockIdx.y;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
    uint32_t* ref_t = ref + (size_t)t * g.B;
    if (!on[t]) {  // uniform: every row is a coded row
        for (uint32_t row = wave_global * 64 + lane; row < g.B; row += rows_grid * 64) ref_t[row] = row;
        return;
    }
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint64_t* kk = keys + (size_t)t * M;
    for (uint32_t row0 = wave_global * kRmRows; row0 < g.B; row0 += rows_grid * kRmRows) {
        uint32_t own = 0xFFFFFFFFu;
        {
            const uint32_t row = row0 + lane;
            if (lane < kRmRows && row < g.B) {
                const uint64_t hsh = rowhash[(size_t)t * g.B + row];
                uint32_t pos = (uint32_t)(hsh >> 20) & (M - 1u);
                for (uint32_t probe_n = 0; probe_n < M; ++probe_n) {
                    if (kk[pos] == hsh) { own = owner[(size_t)t * M + pos]; break; }
                    pos = (pos + 1u) & (M - 1u);
                }
            }
        }
        uint32_t ownk[kRmRows];
        bool need[kRmRows];
#pragma unroll
        for (uint32_t c = 0; c < kRmRows; ++c) {
            ownk[c] = (uint32_t)__shfl((int)own, (int)c, 64);
            const uint32_t row = row0 + c;
            need[c] = row < g.B && ownk[c] < row;  // (an owner is never a later row; "nobody" cannot happen after pass 1)
        }
        // comparisons (uniform conditions: every lane holds the same ownk[] and need[])
        bool differ[kRmRows];
#pragma unroll
        for (uint32_t c = 0; c < kRmRows; ++c) differ[c] = false;
        for (uint32_t e = lane; e < g.D; e += 64) {
#pragma unroll
            for (uint32_t c = 0; c < kRmRows; ++c) {
                if (!need[c]) continue;
                const uint64_t a = rm_identity<F16>(tab, (row0 + c) * g.D + e, q, Rf, (int)g.R);
                const uint64_t b = rm_identity<F16>(tab, ownk[c] * g.D + e, q, Rf, (int)g.R);
                differ[c] = differ[c] || a != b;
            }
        }
#pragma unroll
        for (uint32_t c = 0; c < kRmRows; ++c) {
            const uint32_t row = row0 + c;
            if (row >= g.B) continue;  // uniform
            const bool same = need[c] && __ballot(differ[c]) == 0ull;
            if (lane == 0) ref_t[row] = same ? ownk[c] : row;
        }
    }
}

hipError_t launch_row_match(const Geom& g, const void* payload, const Ws& w, hipStream_t s) {
    const uint32_t M = w.rm_M;
    const size_t n_slots = (size_t)g.T * M;
    hipLaunchKernelGGL(k_rm_clear, dim3((uint32_t)std::min<size_t>((n_slots + 255) / 256, 4096)), dim3(256), 0, s, w.rm_keys,
                       w.rm_owner, n_slots);
    const uint32_t blocks_x = std::min<uint32_t>((g.B + 4 * kRmRows - 1) / (4 * kRmRows), 32u);
    const uint32_t rows_grid = blocks_x * 4;
    dim3 grid(blocks_x, g.T), block(256);
    if (g.dtype == DLC_F16) {
        hipLaunchKernelGGL(k_rm_hash<true>, grid, block, 0, s, payload, g, w.qp, w.rm_on, M, w.rm_keys, w.rm_owner, w.rm_hash, rows_grid);
        hipLaunchKernelGGL(k_rm_owner<true>, grid, block, 0, s, payload, g, w.qp, w.rm_on, M, w.rm_keys, w.rm_owner, w.rm_hash, w.rm_ref, rows_grid);
    } else {
        hipLaunchKernelGGL(k_rm_hash<false>, grid, block, 0, s, payload, g, w.qp, w.rm_on, M, w.rm_keys, w.rm_owner, w.rm_hash, rows_grid);
        hipLaunchKernelGGL(k_rm_owner<false>, grid, block, 0, s, payload, g, w.qp, w.rm_on, M, w.rm_keys, w.rm_owner, w.rm_hash, w.rm_ref, rows_grid);
    }
    return hipGetLastError();
}

}  // namespace dlc
