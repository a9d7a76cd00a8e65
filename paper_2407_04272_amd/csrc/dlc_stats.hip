// Statistics reduction for gfx950: per-table value range and exact distinct-row counts of the raw rows
// and of the rows quantised at a probe bound (the two counts of the Homogenization Index, Eq. 1).
//
// k_stats_init sets an attempt up.  k_stats_hash: two 64-bit hashes per row (raw bits; symbols at the probe bound) and the range.
// The row sets (dlc_rowmatch.hip: the rows of a table divided among work-groups by hash, open-addressing sets in
// LDS, the smallest row index of a hash owns it) give every row the owner of its hash and count the owners.
// k_stats_verify: every row that is not an owner is compared with its owner element by element, so a hash
// collision between different rows is detected (the host then repeats the reduction with another hash salt) and
// the counts are exact.
#include <algorithm>

#include "dlc_internal.h"

#ifndef DLC_STATS_BLOCKS
#define DLC_STATS_BLOCKS 32
#endif

namespace dlc {

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ uint32_t mix32(uint32_t z) {
    z ^= z >> 16; z *= 0x85EBCA6Bu;
    z ^= z >> 13; z *= 0xC2B2AE35u;
    z ^= z >> 16;
    return z;
}

// float <-> unsigned with the same ordering
__device__ __forceinline__ uint32_t ord_enc(float f) {
    uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

template <bool F16>
__device__ __forceinline__ float elem_value(uint32_t raw) {
    if constexpr (F16) return __half2float(__ushort_as_half((unsigned short)raw));
    else return __uint_as_float(raw);
}

constexpr uint32_t kStSlab = 16;            // words of a row that the hash kernel holds in LDS at a time
constexpr uint32_t kStPitch = kStSlab + 1u; // odd: the lanes of a wavefront walk 64 different rows without bank conflicts
constexpr uint32_t kStMult = 4;             // words per position in the multiplier table
constexpr uint32_t kStSteps = 2;            // row sets of a wavefront whose loads the verify kernel issues back to back

struct StatAcc {
    uint32_t r[2], q[2];  // multilinear sums modulo 2^32: raw bits, symbols
    float fmn, fmx;       // range of the finite values (+inf, -inf: none yet)
    uint32_t mn, mx;      // the same as order-preserving integers, at the end
};

// one element: range, symbol at the probe bound, and its share of the four sums.  m: the position's four 24-bit
// multipliers (the same for all lanes: they come through scalar loads); raw bits go in as two 16-bit halves.
// No branches: the loop around this is meant to be scheduled as one block.
template <bool F16>
__device__ __forceinline__ void st_element(uint32_t raw, const uint4& m, const QParam& q, float Rf, int R, StatAcc& A) {
    const float x = elem_value<F16>(raw);
    const bool finite = __builtin_fabsf(x) < __builtin_inff();
    const float xf = finite ? x : __builtin_nanf("");  // minimum and maximum pass over a NaN operand
    A.fmn = __builtin_fminf(A.fmn, xf);
    A.fmx = __builtin_fmaxf(A.fmx, xf);
    const uint32_t c = quant_symbol<F16>(x, q, Rf, R);
    if constexpr (F16) {
        A.r[0] += __umul24(raw, m.x);
        A.r[1] += __umul24(raw, m.y);
    } else {
        const uint32_t lo = raw & 0xFFFFu, hi = raw >> 16;
        A.r[0] += __umul24(lo, m.x) + __umul24(hi, m.z);
        A.r[1] += __umul24(lo, m.y) + __umul24(hi, m.w);
    }
    A.q[0] += __umul24(c, m.x);
    A.q[1] += __umul24(c, m.w);
}

// a word of the staged row at word position p (PACK elements)
template <bool F16, uint32_t PACK>
__device__ __forceinline__ void st_word(uint32_t w, uint32_t p, const uint4* __restrict__ mult, const QParam& q, float Rf, int R,
                                        StatAcc& A) {
    if constexpr (PACK == 2) {
        st_element<F16>(w & 0xFFFFu, mult[2u * p], q, Rf, R, A);
        st_element<F16>(w >> 16, mult[2u * p + 1u], q, Rf, R, A);
    } else {
        st_element<F16>(w, mult[p], q, Rf, R, A);
    }
}

}  // namespace

// start of an attempt: the multipliers of every position of a row for this attempt's salt; the tables' range words
// ("none yet"), the counts of distinct rows and the collision counter cleared
__global__ __launch_bounds__(256) void k_stats_init(uint32_t* mult, uint32_t D, uint32_t salt, uint32_t* minmax, uint32_t* unique,
                                                    uint32_t T, Ctrl* ctrl) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < D * kStMult) {
        const uint32_t e = i / kStMult, k = i % kStMult;
        mult[i] = mix32((e * kStMult + k + 1u) * 0x9E3779B1u + salt) & 0xFFFFFFu;
    }
    if (i < 2u * T) {
        minmax[i] = (i & 1u) ? 0u : 0xFFFFFFFFu;
        unique[i] = 0u;
    }
    if (i == 0) ctrl->collide = 0u;
}

// pass 1, a lane per row.  A wavefront takes 64 consecutive rows, loads kStSlab words of each at a time (PL words
// per lane and load: 16 bytes where the row length allows) into LDS with an odd pitch, and every lane then walks
// its own row there.  PACK: elements per word (2: binary16 pairs; a binary16 row of odd length is loaded element
// by element, one per word).
template <bool F16, uint32_t PACK, uint32_t PL>
__global__ __launch_bounds__(256) void k_stats_hash(const void* payload, Geom g, const QParam* probe, const uint4* __restrict__ mult,
                                                    uint64_t* rowhash, uint32_t* minmax, uint32_t waves_grid) {
    __shared__ uint32_t stage[4][64 * kStPitch];
    const uint32_t t = blockIdx.y;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t wave_global = blockIdx.x * 4 + wave;
    const QParam q = probe[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t Wd = g.D / PACK;  // words per row
    uint32_t* st = stage[wave];
    StatAcc A;
    A.fmn = __builtin_inff();
    A.fmx = -__builtin_inff();
    A.r[0] = A.r[1] = A.q[0] = A.q[1] = 0u;
    constexpr uint32_t kLoads = 64u * kStSlab / (64u * PL);  // loads per lane and slab
    for (uint32_t row0 = wave_global * 64u; row0 < g.B; row0 += waves_grid * 64u) {
        const uint32_t nrows = min(64u, g.B - row0);
        A.r[0] = A.r[1] = A.q[0] = A.q[1] = 0u;
        for (uint32_t p0 = 0; p0 < Wd; p0 += kStSlab) {
            const uint32_t sw = min(kStSlab, Wd - p0);          // words of every row in this slab
            const uint32_t npr = sw / PL, total = nrows * npr;  // pieces per row (PL == 4 only where Wd % 4 == 0), pieces in all
            const float inv = 1.0f / (float)npr;
            uint32_t v[kLoads][PL], dst[kLoads];
#pragma unroll
            for (uint32_t u = 0; u < kLoads; ++u) {
                const uint32_t i = u * 64u + lane;
                dst[u] = 0xFFFFFFFFu;
                if (i < total) {
                    const uint32_t r = (uint32_t)(((float)i + 0.5f) * inv);  // i / npr, exact for these sizes
                    const uint32_t c = (i - r * npr) * PL;
                    const size_t word = (size_t)(row0 + r) * Wd + p0 + c;
                    dst[u] = r * kStPitch + c;
                    if constexpr (PL == 4) {
                        const uint4 x = *reinterpret_cast<const uint4*>(tab + word * 4u);
                        v[u][0] = x.x; v[u][1] = x.y; v[u][2] = x.z; v[u][3] = x.w;
                    } else if constexpr (F16 && PACK == 1) {
                        v[u][0] = reinterpret_cast<const uint16_t*>(tab)[word];
                    } else {
                        v[u][0] = reinterpret_cast<const uint32_t*>(tab)[word];
                    }
                }
            }
#pragma unroll
            for (uint32_t u = 0; u < kLoads; ++u) {
                if (dst[u] != 0xFFFFFFFFu) {
#pragma unroll
                    for (uint32_t k = 0; k < PL; ++k) st[dst[u] + k] = v[u][k];
                }
            }
            // the words come from other lanes of this wavefront: its LDS accesses complete in order, the compiler
            // must keep them in order too
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (lane < nrows) {
                const uint32_t* mine = st + lane * kStPitch;
                const uint32_t full = sw & ~3u;
                for (uint32_t c0 = 0; c0 < full; c0 += 4u) {  // (position and multipliers: the same for all lanes)
                    uint32_t w[4];
#pragma unroll
                    for (uint32_t k = 0; k < 4; ++k) w[k] = mine[c0 + k];
#pragma unroll
                    for (uint32_t k = 0; k < 4; ++k) st_word<F16, PACK>(w[k], p0 + c0 + k, mult, q, Rf, (int)g.R, A);
                }
                for (uint32_t c = full; c < sw; ++c) st_word<F16, PACK>(mine[c], p0 + c, mult, q, Rf, (int)g.R, A);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        const uint32_t row = row0 + lane;
        if (row < g.B) {
            rowhash[(size_t)t * g.B + row] = mix64(((uint64_t)A.r[1] << 32) | A.r[0]);
            rowhash[((size_t)g.T + t) * g.B + row] = mix64((((uint64_t)A.q[1] << 32) | A.q[0]) ^ 0x5555555555555555ull);
        }
    }
    // the range as order-preserving integers
    A.mn = A.fmn == __builtin_inff() ? 0xFFFFFFFFu : ord_enc(A.fmn);
    A.mx = A.fmx == -__builtin_inff() ? 0u : ord_enc(A.fmx);
    uint32_t mn = A.mn, mx = A.mx;
    for (int o = 32; o > 0; o >>= 1) {
        mn = min(mn, (uint32_t)__shfl_xor(mn, o, 64));
        mx = max(mx, (uint32_t)__shfl_xor(mx, o, 64));
    }
    if (lane == 0) {
        atomicMin(&minmax[2 * t], mn);
        atomicMax(&minmax[2 * t + 1], mx);
    }
}

namespace {

// a lane's piece of a row: NW words (16 bytes where the row length allows, else one element in one word)
template <uint32_t NW>
struct StPiece { uint32_t v[NW]; };

template <bool F16, uint32_t NW>
__device__ __forceinline__ StPiece<NW> st_load_piece(const uint8_t* tab, size_t piece) {
    StPiece<NW> r;
    if constexpr (NW == 4) {
        const uint4 x = *reinterpret_cast<const uint4*>(tab + piece * 16u);
        r.v[0] = x.x; r.v[1] = x.y; r.v[2] = x.z; r.v[3] = x.w;
    } else if constexpr (F16) {
        r.v[0] = reinterpret_cast<const uint16_t*>(tab)[piece];
    } else {
        r.v[0] = reinterpret_cast<const uint32_t*>(tab)[piece];
    }
    return r;
}

// do two words (of different bits) hold elements with different symbols?
template <bool F16, uint32_t NW>
__device__ __forceinline__ bool st_symbols_differ(uint32_t a, uint32_t b, const QParam& q, float Rf, int R) {
    if constexpr (F16 && NW == 4) {  // two elements per word
        return quant_symbol<true>(elem_value<true>(a & 0xFFFFu), q, Rf, R) != quant_symbol<true>(elem_value<true>(b & 0xFFFFu), q, Rf, R) ||
               quant_symbol<true>(elem_value<true>(a >> 16), q, Rf, R) != quant_symbol<true>(elem_value<true>(b >> 16), q, Rf, R);
    } else {
        return quant_symbol<F16>(elem_value<F16>(a), q, Rf, R) != quant_symbol<F16>(elem_value<F16>(b), q, Rf, R);
    }
}

}  // namespace

// pass 2: every row that does not own its hash must equal the owner: in its bits for the raw rows, in its symbols for
// the quantised rows (only the elements whose bits differ need the quantiser).  A row is the work of a team of
// 2^logL lanes, the smallest power of two that covers the row's pieces (64 at most: longer rows take several
// trips); a wavefront works on 64 rows per trip, 64 >> logL at a time.  own: [2][T][B], raw then quantised.
template <bool F16, uint32_t NW>
__global__ __launch_bounds__(256) void k_stats_verify(const void* payload, Geom g, const QParam* probe, const uint32_t* own,
                                                      Ctrl* ctrl, uint32_t waves_grid, uint32_t logL) {
    const uint32_t t = blockIdx.y;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
    const QParam q = probe[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t W = NW == 4 ? (uint32_t)((size_t)g.D * g.es / 16u) : g.D;  // pieces per row
    const uint32_t L = 1u << logL, sub = lane & (L - 1u), team = lane >> logL, rps = 64u >> logL;
    bool differ = false;
    for (uint32_t row0 = wave_global * 64u; row0 < g.B; row0 += waves_grid * 64u) {
        uint32_t or_mine = 0xFFFFFFFFu, oq_mine = 0xFFFFFFFFu;  // lane j: the owners of row row0 + j's two hashes
        {
            const uint32_t row = row0 + lane;
            if (row < g.B) {
                or_mine = own[(size_t)t * g.B + row];
                oq_mine = own[((size_t)g.T + t) * g.B + row];
            }
        }
        for (uint32_t s0 = 0; s0 < L; s0 += kStSteps) {  // L steps of rps rows make 64 rows
            uint32_t orr[kStSteps], oq[kStSteps];
            bool need_r[kStSteps], need_q[kStSteps];
#pragma unroll
            for (uint32_t s = 0; s < kStSteps; ++s) {
                const uint32_t r = (s0 + s) * rps + team;
                orr[s] = (uint32_t)__shfl((int)or_mine, (int)(r & 63u), 64);
                oq[s] = (uint32_t)__shfl((int)oq_mine, (int)(r & 63u), 64);
                const bool live = s0 + s < L && row0 + r < g.B;
                need_r[s] = live && orr[s] < row0 + r;  // (an owner is never a later row)
                need_q[s] = live && oq[s] < row0 + r;
            }
            for (uint32_t p = sub; p < W; p += L) {
                StPiece<NW> a[kStSteps], br[kStSteps], bq[kStSteps];
#pragma unroll
                for (uint32_t s = 0; s < kStSteps; ++s) {
                    const uint32_t row = row0 + (s0 + s) * rps + team;
                    if (need_r[s] || need_q[s]) a[s] = st_load_piece<F16, NW>(tab, (size_t)row * W + p);
                    if (need_r[s]) br[s] = st_load_piece<F16, NW>(tab, (size_t)orr[s] * W + p);
                    if (need_q[s] && !(need_r[s] && oq[s] == orr[s])) bq[s] = st_load_piece<F16, NW>(tab, (size_t)oq[s] * W + p);
                }
#pragma unroll
                for (uint32_t s = 0; s < kStSteps; ++s) {
                    if (need_r[s]) {
#pragma unroll
                        for (uint32_t k = 0; k < NW; ++k) differ |= a[s].v[k] != br[s].v[k];
                    }
                    if (need_q[s]) {
                        const bool shared = need_r[s] && oq[s] == orr[s];
#pragma unroll
                        for (uint32_t k = 0; k < NW; ++k) {
                            const uint32_t b = shared ? br[s].v[k] : bq[s].v[k];
                            if (a[s].v[k] != b) differ |= st_symbols_differ<F16, NW>(a[s].v[k], b, q, Rf, (int)g.R);
                        }
                    }
                }
            }
        }
    }
    if (__ballot(differ) != 0ull && lane == 0) atomicAdd(&ctrl->collide, 1u);
}

hipError_t launch_stats(const Geom& g, const void* payload, const QParam* probe, const Ws& w, uint32_t salt, hipStream_t s) {
    // few, long-running work-groups per table: every wavefront ends with atomics on its table's two range words
    const uint32_t blocks_x = std::min<uint32_t>((g.B + 255u) / 256u, DLC_STATS_BLOCKS);  // a wavefront takes 64 rows at a time
    const uint32_t waves_grid = blocks_x * 4;
    dim3 grid(blocks_x, g.T), block(256);
    hipLaunchKernelGGL(k_stats_init, dim3((std::max(g.D * kStMult, 2u * g.T) + 255u) / 256u), block, 0, s, w.st_mult, g.D, salt,
                       w.st_minmax, w.st_unique, g.T, w.ctrl);
#define DLC_ST_HASH(FF, PK, PL) hipLaunchKernelGGL((k_stats_hash<FF, PK, PL>), grid, block, 0, s, payload, g, probe, reinterpret_cast<const uint4*>(w.st_mult), w.rowhash, w.st_minmax, waves_grid)
    if (g.dtype == DLC_F16) {
        if (g.D % 8u == 0u) DLC_ST_HASH(true, 2, 4);
        else if (g.D % 2u == 0u) DLC_ST_HASH(true, 2, 1);
        else DLC_ST_HASH(true, 1, 1);
    } else {
        if (g.D % 4u == 0u) DLC_ST_HASH(false, 1, 4);
        else DLC_ST_HASH(false, 1, 1);
    }
#undef DLC_ST_HASH
    hipError_t e = launch_row_sets(g, 2u, nullptr, w.rowhash, w.st_own, w.st_unique, w.ctrl, s);
    if (e != hipSuccess) return e;
    const bool vec = ((size_t)g.D * g.es) % 16u == 0u;
    const uint32_t pieces = vec ? (uint32_t)((size_t)g.D * g.es / 16u) : g.D;
    uint32_t logL = 0;
    while (logL < 6 && (1u << logL) < pieces) ++logL;
#define DLC_ST_VERIFY(FF, NW) hipLaunchKernelGGL((k_stats_verify<FF, NW>), grid, block, 0, s, payload, g, probe, w.st_own, w.ctrl, waves_grid, logL)
    if (g.dtype == DLC_F16) { if (vec) DLC_ST_VERIFY(true, 4); else DLC_ST_VERIFY(true, 1); }
    else { if (vec) DLC_ST_VERIFY(false, 4); else DLC_ST_VERIFY(false, 1); }
#undef DLC_ST_VERIFY
    return hipGetLastError();
}

}  // namespace dlc
