// Row matching for gfx950 (the vector-based LZ step of Section III-D: the fixed pattern is one embedding vector).
// For every row of a table: the first row of the batch with the same content after quantisation (all symbols
// equal and, where a symbol is the escape, the raw bits too).  Rows that have an earlier equal are not coded by
// the kernels that follow; they are stored as references.
//
// Three kernels, after the histogram kernel and on its symbol plane: a 64-bit hash per row; per table, sets of the
// rows by hash, kept in LDS (the table's rows are divided among several work-groups by their hashes, so no two
// work-groups ever meet in a set and no atomic leaves the LDS), the smallest row index of a hash owning it; then
// every other row is compared with the owner of its hash element by element.  A row whose hash meets a different
// row's (three multilinear sums modulo 2^32 with 24-bit multipliers: 2^-48 for a pair of rows at worst, far less
// for most) is looked up the long way, among the earlier rows with that hash, so the references are those of the
// definition (the first row with the content) whatever the hashes do.
#include <algorithm>

#include "dlc_internal.h"
#include "dlc_codec_dev.h"

namespace dlc {

namespace {

__device__ __forceinline__ uint64_t rm_mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__host__ __device__ __forceinline__ uint32_t rm_mix32(uint32_t z) {
    z ^= z >> 16; z *= 0x85EBCA6Bu;
    z ^= z >> 13; z *= 0xC2B2AE35u;
    z ^= z >> 16;
    return z;
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

// is one of the four bytes 254 or 255 (the plane's "escape" and "outside the window": what the element is, its raw
// bits or its symbol, is in the payload)?
__device__ __forceinline__ bool rm_has255(uint32_t w) {
    const uint32_t x = ~(w | 0x01010101u);
    return ((x - 0x01010101u) & ~x & 0x80808080u) != 0u;
}

// adds the piece's two halves to the three sums (multilinear, modulo 2^32); m: the 24-bit multipliers of the
// piece's position in the row, two per sum
__device__ __forceinline__ void rm_add_piece(uint32_t w, const uint4& m03, const uint2& m45, uint32_t a[3]) {
    const uint32_t lo = w & 0xFFFFu, hi = w >> 16;
    a[0] += __umul24(lo, m03.x) + __umul24(hi, m03.y);
    a[1] += __umul24(lo, m03.z) + __umul24(hi, m03.w);
    a[2] += __umul24(lo, m45.x) + __umul24(hi, m45.y);
}

// what an element outside the window adds to the three sums: by what it is and where it is
__device__ __forceinline__ void rm_add_other(uint64_t id, uint32_t e, uint32_t a[3]) {
    const uint32_t z = rm_mix32((uint32_t)id + 0x9E3779B9u * (e + 1u)) ^ ((id >> 32) ? 0x7F4A7C15u : 0u);
    a[0] += z;
    a[1] += rm_mix32(z);
    a[2] += rm_mix32(z ^ 0x5BD1E995u);
}

constexpr uint32_t kRmSteps = 4;  // row sets of a wavefront whose loads are issued back to back
constexpr uint32_t kRmSlab = 32;   // pieces of a row that pass 1 holds in LDS at a time
constexpr uint32_t kRmPitch = kRmSlab + 1u;

}  // namespace

// The hash and the verify kernel read the symbol plane the histogram kernel has written (one byte per element: the
// symbol's window index, 254 for an escape, 255 for a symbol outside the window), four bytes (a piece) at a time.
// An element with index 254 or 255 is looked up in the payload: the raw bits of an escape, or the symbol.

// pass 1: hash of every row, a lane per row.  A wavefront takes 64 consecutive rows: it loads their pieces as
// they lie in memory (16 bytes per lane where the row length allows), kRmSlab pieces of each row at a time, into LDS
// with an odd pitch, and every lane then walks its own row there; the multipliers of a position are the same
// for all lanes.
template <bool F16>
__global__ __launch_bounds__(256) void k_rm_hash(const void* payload, Geom g, const QParam* qp, const uint8_t* on,
                                                 uint64_t* rowhash, const uint8_t* sym_plane,
                                                 const uint32_t* __restrict__ mult, uint32_t waves_grid) {
    __shared__ uint32_t stage[4][64 * kRmPitch];
    const uint32_t t = blockIdx.y;
    if (!on[t]) return;  // uniform: the table is coded row by row as it is
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t wave_global = blockIdx.x * 4 + wave;
    const uint32_t W = g.D / 4u;
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    const uint32_t* plane = reinterpret_cast<const uint32_t*>(sym_plane + (size_t)t * plane_stride(g));
    uint32_t* st = stage[wave];
    for (uint32_t row0 = wave_global * 64u; row0 < g.B; row0 += waves_grid * 64u) {
        const uint32_t nrows = min(64u, g.B - row0);
        uint32_t a[3] = {0u, 0u, 0u};
        for (uint32_t p0 = 0; p0 < W; p0 += kRmSlab) {
            const uint32_t sw = min(kRmSlab, W - p0);  // pieces of every row in this slab
            const uint32_t total = nrows * sw;         // 2048 at most
            if (sw == W && (W & 3u) == 0u) {  // whole rows, one after the other in memory, 16-byte pieces
                const uint4* src = reinterpret_cast<const uint4*>(plane + (size_t)row0 * W);
                const uint32_t n4 = total / 4u;
                const float inv = 1.0f / (float)W;
                for (uint32_t k0 = 0; k0 < n4; k0 += 64u * 8u) {
                    uint4 v[8];
#pragma unroll
                    for (uint32_t u = 0; u < 8; ++u) {
                        const uint32_t i = k0 + u * 64u + lane;
                        v[u] = i < n4 ? src[i] : make_uint4(0, 0, 0, 0);
                    }
#pragma unroll
                    for (uint32_t u = 0; u < 8; ++u) {
                        const uint32_t i = k0 + u * 64u + lane;
                        if (i < n4) {
                            const uint32_t idx = i * 4u;
                            const uint32_t r = (uint32_t)(((float)idx + 0.5f) * inv);  // idx / W, exact for these sizes
                            uint32_t* d = st + idx + r * (kRmPitch - W);               // row r, piece idx - r * W
                            d[0] = v[u].x; d[1] = v[u].y; d[2] = v[u].z; d[3] = v[u].w;
                        }
                    }
                }
            } else {
                const float inv = 1.0f / (float)sw;
                for (uint32_t i = lane; i < total; i += 64u) {
                    const uint32_t r = (uint32_t)(((float)i + 0.5f) * inv), c = i - r * sw;
                    st[r * kRmPitch + c] = plane[(size_t)(row0 + r) * W + p0 + c];
                }
            }
            // the pieces come from other lanes of this wavefront: its LDS accesses complete in order, the compiler
            // must keep them in order too
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (lane < nrows) {
                const uint32_t* mine = st + lane * kRmPitch;
                for (uint32_t c0 = 0; c0 < sw; c0 += 4u) {  // (position and multipliers: the same for all lanes)
                    uint32_t w[4];
#pragma unroll
                    for (uint32_t k = 0; k < 4; ++k) w[k] = c0 + k < sw ? mine[c0 + k] : 0u;
                    bool other = false;
#pragma unroll
                    for (uint32_t k = 0; k < 4; ++k) {
                        const uint32_t p = min(p0 + c0 + k, W - 1u);  // (a piece past the row's end is 0 and adds nothing)
                        const uint4 m03 = *reinterpret_cast<const uint4*>(mult + 8u * p);
                        const uint2 m45 = *reinterpret_cast<const uint2*>(mult + 8u * p + 4u);
                        rm_add_piece(w[k], m03, m45, a);
                        other = other || rm_has255(w[k]);
                    }
                    if (other) {  // rare
                        for (uint32_t k = 0; k < 4; ++k) {
                            for (uint32_t v = 0; v < 4; ++v) {
                                if (((w[k] >> (8u * v)) & 255u) < kWinEsc) continue;
                                const uint32_t e = (p0 + c0 + k) * 4u + v;
                                rm_add_other(rm_identity<F16>(tab, (row0 + lane) * g.D + e, q, Rf, (int)g.R), e, a);
                            }
                        }
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        const uint32_t row = row0 + lane;
        if (row < g.B)
            rowhash[(size_t)t * g.B + row] = rm_mix64((((uint64_t)a[1] << 32) | a[0]) + (uint64_t)a[2] * 0x9E3779B97F4A7C15ull);
    }
}

// the sets: work-group (part, t, set) takes the rows of table t whose hashes' top bits say `part`, puts them into an
// open-addressing set in LDS (a slot holds a row index; the hash of the row that sits there is read from memory,
// and only rows with that hash ever replace it, the smaller index winning), and then looks every one of its rows
// up again: own[row] = the smallest row index with the row's hash.  n_slots (a power of two) is the batch size or
// more whenever that fits the LDS, so the set cannot fill up; for larger batches a work-group's share of the rows
// is half the slots or less, and where a set does fill up all the same (hashes that crowd into one share), the rows that
// found no slot are their own owners (coded rows, for row matching), and ctrl, if given, gets an error (the
// statistics want exact counts).  rowhash and own: [sets][T][B]; on (optional): tables to skip; unique (optional):
// [T][sets] counts of the rows that own their hash.
__global__ __launch_bounds__(1024) void k_rm_sets(Geom g, const uint8_t* on, const uint64_t* rowhash, uint32_t* own,
                                                  uint32_t n_slots, uint32_t parts, uint32_t* unique, Ctrl* ctrl) {
    extern __shared__ __align__(16) uint32_t slot[];
    __shared__ uint32_t s_owners;
    const uint32_t part = blockIdx.x, t = blockIdx.y, set = blockIdx.z, tid = threadIdx.x;
    if (on && !on[t]) return;  // uniform
    constexpr uint32_t kEmpty = 0xFFFFFFFFu;
    constexpr uint32_t kBatch = 4;  // hashes a thread loads back to back
    for (uint32_t k = tid; k < n_slots; k += 1024) slot[k] = kEmpty;
    if (tid == 0) s_owners = 0u;
    __syncthreads();
    const uint64_t* rh = rowhash + ((size_t)set * g.T + t) * g.B;
    uint32_t* own_t = own + ((size_t)set * g.T + t) * g.B;
    volatile uint32_t* vslot = slot;
    for (uint32_t r0 = tid; r0 < g.B; r0 += 1024u * kBatch) {
        uint64_t h[kBatch];
#pragma unroll
        for (uint32_t k = 0; k < kBatch; ++k) h[k] = r0 + k * 1024u < g.B ? rh[r0 + k * 1024u] : 0ull;
#pragma unroll
        for (uint32_t k = 0; k < kBatch; ++k) {
            const uint32_t row = r0 + k * 1024u;
            if (row >= g.B || ((uint32_t)(h[k] >> 52) & (parts - 1u)) != part) continue;
            uint32_t pos = (uint32_t)(h[k] >> 20) & (n_slots - 1u);
            bool placed = false;
            for (uint32_t probe_n = 0; probe_n < n_slots; ++probe_n) {
                uint32_t cur = vslot[pos];
                if (cur == kEmpty) {
                    cur = atomicCAS(&slot[pos], kEmpty, row);
                    if (cur == kEmpty) { placed = true; break; }
                }
                if (rh[cur] == h[k]) {
                    atomicMin(&slot[pos], row);
                    placed = true;
                    break;
                }
                pos = (pos + 1u) & (n_slots - 1u);
            }
            if (!placed && ctrl) set_status(ctrl, DLC_ESTATE);
        }
    }
    __syncthreads();
    uint32_t owners = 0;
    for (uint32_t r0 = tid; r0 < g.B; r0 += 1024u * kBatch) {
        uint64_t h[kBatch];
#pragma unroll
        for (uint32_t k = 0; k < kBatch; ++k) h[k] = r0 + k * 1024u < g.B ? rh[r0 + k * 1024u] : 0ull;
#pragma unroll
        for (uint32_t k = 0; k < kBatch; ++k) {
            const uint32_t row = r0 + k * 1024u;
            if (row >= g.B || ((uint32_t)(h[k] >> 52) & (parts - 1u)) != part) continue;
            uint32_t o = row;
            uint32_t pos = (uint32_t)(h[k] >> 20) & (n_slots - 1u);
            for (uint32_t probe_n = 0; probe_n < n_slots; ++probe_n) {
                const uint32_t cur = vslot[pos];
                if (cur == kEmpty) break;
                if (cur == row || rh[cur] == h[k]) { o = cur; break; }
                pos = (pos + 1u) & (n_slots - 1u);
            }
            own_t[row] = o;
            owners += o == row ? 1u : 0u;
        }
    }
    if (unique) {  // uniform
        for (int o = 32; o > 0; o >>= 1) owners += (uint32_t)__shfl_xor((int)owners, o, 64);
        if ((tid & 63u) == 0u && owners) atomicAdd(&s_owners, owners);
        __syncthreads();
        if (tid == 0 && s_owners) atomicAdd(&unique[(size_t)t * gridDim.z + set], s_owners);
    }
}

// pass 2: ref[row] = the owner of the row's hash if the two rows are equal element by element, else the row itself.
// The elements of a row that refers to another leave the table's counts again (the histogram kernel has counted
// every row) and get index 253 in the plane, which the encode kernel's table maps to no bits at all.  Only rows
// that nobody compares with are changed: an owner is never such a row.
// A lane holds a piece of PW words of the plane (16 bytes where the row length allows, else 4); a row is the work
// of a team of 2^logL lanes, the smallest power of two that covers the row's pieces (64 at most: longer rows take
// several trips); a wavefront works on 64 rows per trip: 64 >> logL at a time, in 2^logL steps, kRmSteps of them
// with their loads issued back to back.
template <uint32_t PW>
struct RmPiece { uint32_t v[PW]; };

template <uint32_t PW>
__device__ __forceinline__ RmPiece<PW> rm_load_piece(const uint32_t* plane, size_t piece) {
    RmPiece<PW> r;
    if constexpr (PW == 4) {
        const uint4 q = *reinterpret_cast<const uint4*>(plane + piece * 4u);
        r.v[0] = q.x; r.v[1] = q.y; r.v[2] = q.z; r.v[3] = q.w;
    } else {
        r.v[0] = plane[piece];
    }
    return r;
}

template <bool F16, uint32_t PW>
__global__ __launch_bounds__(256) void k_rm_owner(const void* payload, Geom g, const QParam* qp, const uint8_t* on,
                                                  const uint32_t* rowown, const uint64_t* rowhash, uint32_t* ref, uint8_t* sym_plane,
                                                  uint32_t* hist, uint32_t waves_grid, uint32_t logL) {
    extern __shared__ __align__(16) uint32_t lh[];  // what to take off the counts: window [kWinBins + 1][kWinCopies] | exact [K]
    const uint32_t t = blockIdx.y;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave_global = blockIdx.x * 4 + (tid >> 6);
    uint32_t* ref_t = ref + (size_t)t * g.B;
    if (!on[t]) {  // uniform: every row is a coded row
        for (uint32_t row = wave_global * 64 + lane; row < g.B; row += waves_grid * 64) ref_t[row] = row;
        return;
    }
    const uint32_t n_words = (kWinBins + 1u) * kWinCopies + g.K;
    {
        uint4* z = reinterpret_cast<uint4*>(lh);
        for (uint32_t k = tid; k < (n_words + 3u) / 4u; k += 256) z[k] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    uint32_t* win = lh + (lane & (kWinCopies - 1u));
    uint32_t* exact = lh + (kWinBins + 1u) * kWinCopies;
    const uint32_t L = 1u << logL, sub = lane & (L - 1u), team = lane >> logL, rps = 64u >> logL, W = g.D / (4u * PW);
    const uint64_t teammask = (L == 64u ? ~0ull : ((1ull << L) - 1ull)) << (team * L);
    const QParam q = qp[t];
    const float Rf = (float)g.R;
    const uint8_t* tab = static_cast<const uint8_t*>(payload) + (size_t)t * g.n * g.es;
    uint32_t* plane = reinterpret_cast<uint32_t*>(sym_plane + (size_t)t * plane_stride(g));
    for (uint32_t row0 = wave_global * 64u; row0 < g.B; row0 += waves_grid * 64u) {
        uint32_t own_mine = 0xFFFFFFFFu;  // lane j: the owner of row row0 + j's hash
        {
            const uint32_t row = row0 + lane;
            if (row < g.B) own_mine = rowown[(size_t)t * g.B + row];
        }
        for (uint32_t s0 = 0; s0 < L; s0 += kRmSteps) {  // L steps of rps rows make 64 rows
            uint32_t own[kRmSteps];
            bool need[kRmSteps], differ[kRmSteps];
            RmPiece<PW> w[kRmSteps];  // the row's piece of the last trip (the only one unless a row has more than 64 pieces)
#pragma unroll
            for (uint32_t s = 0; s < kRmSteps; ++s) {
                const uint32_t r = (s0 + s) * rps + team;
                own[s] = (uint32_t)__shfl((int)own_mine, (int)(r & 63u), 64);
                need[s] = s0 + s < L && row0 + r < g.B && own[s] < row0 + r;  // (an owner is never a later row)
                differ[s] = false;
#pragma unroll
                for (uint32_t k = 0; k < PW; ++k) w[s].v[k] = 0u;
            }
            for (uint32_t p = sub; p < W; p += L) {
                RmPiece<PW> b[kRmSteps];
#pragma unroll
                for (uint32_t s = 0; s < kRmSteps; ++s) {
                    const uint32_t row = row0 + (s0 + s) * rps + team;
                    if (need[s]) {
                        w[s] = rm_load_piece<PW>(plane, (size_t)row * W + p);
                        b[s] = rm_load_piece<PW>(plane, (size_t)own[s] * W + p);
                    } else {
#pragma unroll
                        for (uint32_t k = 0; k < PW; ++k) w[s].v[k] = b[s].v[k] = 0u;
                    }
                }
#pragma unroll
                for (uint32_t s = 0; s < kRmSteps; ++s) {
                    uint32_t x = 0u;
                    bool other = false;
#pragma unroll
                    for (uint32_t k = 0; k < PW; ++k) {
                        x |= w[s].v[k] ^ b[s].v[k];
                        other = other || rm_has255(w[s].v[k]);
                    }
                    if (x != 0u) differ[s] = true;
                    else if (other) {  // rare: the elements outside the window, by what they are
                        const uint32_t row = row0 + (s0 + s) * rps + team;
                        for (uint32_t k = 0; k < PW; ++k) {
                            for (uint32_t v = 0; v < 4; ++v) {
                                if (((w[s].v[k] >> (8u * v)) & 255u) < kWinEsc) continue;
                                const uint32_t e = (p * PW + k) * 4u + v;
                                if (rm_identity<F16>(tab, row * g.D + e, q, Rf, (int)g.R) != rm_identity<F16>(tab, own[s] * g.D + e, q, Rf, (int)g.R))
                                    differ[s] = true;
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (uint32_t s = 0; s < kRmSteps; ++s) {
                const uint32_t row = row0 + (s0 + s) * rps + team;
                bool same = need[s] && (__ballot(differ[s]) & teammask) == 0ull;  // the same for all lanes of a team
                // A row that is not its hash's owner's equal: two different rows with one hash.  The first earlier row
                // with the row's content, if there is one, has that hash too: the whole wavefront looks through the
                // earlier rows with it, one such row at a time (never expected; slow and plain).
                uint64_t coll = __ballot(need[s] && !same && sub == 0u);
                while (coll != 0ull) {  // uniform over the wavefront
                    const uint32_t leader = (uint32_t)__ffsll((unsigned long long)coll) - 1u;
                    coll &= coll - 1ull;
                    const uint32_t crow = row0 + (s0 + s) * rps + (leader >> logL);
                    const uint64_t h = rowhash[(size_t)t * g.B + crow];
                    uint32_t found = crow;
                    for (uint32_t j0 = 0; j0 < crow && found == crow; j0 += 64u) {
                        const uint32_t j = j0 + lane;
                        uint64_t m = __ballot(j < crow && rowhash[(size_t)t * g.B + j] == h);
                        while (m != 0ull && found == crow) {
                            const uint32_t jj = j0 + (uint32_t)__ffsll((unsigned long long)m) - 1u;
                            m &= m - 1ull;
                            bool d = false;
                            for (uint32_t e = lane; e < g.D; e += 64u)
                                d = d || rm_identity<F16>(tab, crow * g.D + e, q, Rf, (int)g.R) != rm_identity<F16>(tab, jj * g.D + e, q, Rf, (int)g.R);
                            if (__ballot(d) == 0ull) found = jj;
                        }
                    }
                    if (found != crow && team == (leader >> logL)) {
                        own[s] = found;
                        same = true;
                    }
                }
                if (sub == 0 && s0 + s < L && row < g.B) ref_t[row] = same ? own[s] : row;
                if (!same) continue;
                for (uint32_t p = sub; p < W; p += L) {
                    const RmPiece<PW> wv = W <= L ? w[s] : rm_load_piece<PW>(plane, (size_t)row * W + p);
#pragma unroll
                    for (uint32_t k = 0; k < PW; ++k) {
                        if (!rm_has255(wv.v[k])) {
#pragma unroll
                            for (uint32_t v = 0; v < 4; ++v) atomicSub(&win[((wv.v[k] >> (8u * v)) & 255u) * kWinCopies], 1u);
                        } else {
                            for (uint32_t v = 0; v < 4; ++v) {
                                const uint32_t idx = (wv.v[k] >> (8u * v)) & 255u;
                                if (idx < kWinEsc) {
                                    atomicSub(&win[idx * kWinCopies], 1u);
                                } else {
                                    const uint64_t id = rm_identity<F16>(tab, row * g.D + (p * PW + k) * 4u + v, q, Rf, (int)g.R);
                                    atomicSub(&exact[(id >> 32) ? 0u : (uint32_t)id], 1u);
                                }
                            }
                        }
                    }
                    if constexpr (PW == 4) *reinterpret_cast<uint4*>(plane + ((size_t)row * W + p) * 4u) = make_uint4(0xFDFDFDFDu, 0xFDFDFDFDu, 0xFDFDFDFDu, 0xFDFDFDFDu);
                    else plane[(size_t)row * W + p] = 0xFDFDFDFDu;
                }
            }
        }
    }
    __syncthreads();
    // merge (the sums are negative numbers modulo 2^32, and so is what the global counts get added)
    const uint32_t win_lo = win_lo_of(g.R);
    for (uint32_t k = tid; k < g.K; k += 256) {
        uint32_t s = exact[k];
        const uint32_t wi = k - win_lo;
        if (wi < kWinSkip) {
            const uint32_t* row = lh + wi * kWinCopies;
            for (uint32_t c = 0; c < kWinCopies; ++c) s += row[(c + tid) & (kWinCopies - 1u)];
        }
        if (s) atomicAdd(&hist[(size_t)t * g.K + k], s);
    }
}

void row_match_multipliers(uint32_t* mult, uint32_t n_pieces) {
    for (uint32_t p = 0; p < n_pieces; ++p)
        for (uint32_t i = 0; i < 8; ++i) mult[8 * p + i] = i < 6 ? (rm_mix32(p * 6u + i + 1u) & 0xFFFFFFu) : 0u;
}

hipError_t launch_row_sets(const Geom& g, uint32_t n_sets, const uint8_t* on, const uint64_t* rowhash, uint32_t* own,
                           uint32_t* unique, Ctrl* ctrl, hipStream_t s) {
    // slots for the whole batch, 64 KiB at most; about a thousand work-groups in all (32 per table and set at most),
    // and more where a batch is large: a work-group's share of the rows is half its slots or less (up to 32 M rows)
    uint32_t n_slots = 64;
    while (n_slots < g.B && n_slots < 16384u) n_slots <<= 1;
    uint32_t parts = 1;
    while (parts < 32u && parts * g.T * n_sets < 1024u) parts <<= 1;
    while (parts < 4096u && (uint64_t)parts * n_slots < 2ull * g.B) parts <<= 1;
    hipLaunchKernelGGL(k_rm_sets, dim3(parts, g.T, n_sets), dim3(1024), n_slots * 4u, s, g, on, rowhash, own, n_slots, parts,
                       unique, ctrl);
    return hipGetLastError();
}

hipError_t launch_row_match(const Geom& g, const void* payload, const Ws& w, hipStream_t s) {
    const uint32_t pw = g.D % 16u == 0u ? 4u : 1u;  // words of the plane per lane in pass 2
    uint32_t logL = 0;
    while (logL < 6 && (1u << logL) < g.D / (4u * pw)) ++logL;
    const uint32_t blocks_x = std::min<uint32_t>((g.B + 255u) / 256u, 32u);  // a wavefront takes 64 rows at a time
    const uint32_t waves_grid = blocks_x * 4;
    const size_t sm = hist_lds_bytes(g.K);
    dim3 grid(blocks_x, g.T), block(256);
    if (g.dtype == DLC_F16)
        hipLaunchKernelGGL(k_rm_hash<true>, grid, block, 0, s, payload, g, w.qp, w.rm_on, w.rm_hash, w.sym_plane, w.rm_mult, waves_grid);
    else
        hipLaunchKernelGGL(k_rm_hash<false>, grid, block, 0, s, payload, g, w.qp, w.rm_on, w.rm_hash, w.sym_plane, w.rm_mult, waves_grid);
    {
        hipError_t e = launch_row_sets(g, 1u, w.rm_on, w.rm_hash, w.rm_own, nullptr, nullptr, s);
        if (e != hipSuccess) return e;
    }
#define DLC_RM_OWNER(FF, PP) hipLaunchKernelGGL((k_rm_owner<FF, PP>), grid, block, sm, s, payload, g, w.qp, w.rm_on, w.rm_own, w.rm_hash, w.rm_ref, w.sym_plane, w.hist, waves_grid, logL)
    if (g.dtype == DLC_F16) { if (pw == 4u) DLC_RM_OWNER(true, 4); else DLC_RM_OWNER(true, 1); }
    else { if (pw == 4u) DLC_RM_OWNER(false, 4); else DLC_RM_OWNER(false, 1); }
#undef DLC_RM_OWNER
    return hipGetLastError();
}

hipError_t row_match_set_attributes() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k_rm_sets), hipFuncAttributeMaxDynamicSharedMemorySize, 16384 * 4);
}

}  // namespace dlc
