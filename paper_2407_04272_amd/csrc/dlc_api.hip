// Host side of libdlc: context, argument checks, workspace, error-bound controller, C ABI.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <utility>
#include <limits>
#include <mutex>
#include <new>
#include <vector>

#include "dlc_internal.h"

namespace dlc {
hipError_t compress_set_attributes();
hipError_t decompress_set_attributes();

struct Prof {
    int level = 0;
    struct Rec { int slot; hipEvent_t a, b; };
    std::vector<Rec> recs;       // recorded pairs awaiting read-out
    std::vector<hipEvent_t> pool;
    hipEvent_t pending[P_NSLOTS] = {};
    float total_ms[P_NSLOTS] = {};
    int32_t launches[P_NSLOTS] = {};
    hipEvent_t get() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        (void)hipEventCreate(&e);
        return e;
    }
};

void prof_begin(void* p, int slot, hipStream_t s) {
    Prof* pr = static_cast<Prof*>(p);
    hipEvent_t e = pr->get();
    (void)hipEventRecord(e, s);
    pr->pending[slot] = e;
}
void prof_end(void* p, int slot, hipStream_t s) {
    Prof* pr = static_cast<Prof*>(p);
    hipEvent_t e = pr->get();
    (void)hipEventRecord(e, s);
    pr->recs.push_back({slot, pr->pending[slot], e});
}

static const char* kSlotNames[P_NSLOTS] = {"k_hist", "k_codebook", "k_encode", "k_finalize",
                                           "k_decode", "k_encode_carry", "k_post"};
}  // namespace dlc

using namespace dlc;

struct dlc_ctx {
    dlc_config cfg;
    Geom g;
    Ws ws;
    int device = 0;
    bool bounds_set = false;
    uint64_t epoch = 0;
    Prof prof;
    // pinned staging ring for the per-table quantiser parameters (one slot per set_error_bounds call)
    static constexpr int kRing = 16;
    QParam* pin = nullptr;
    hipEvent_t pin_ev[kRing] = {};
    bool pin_used[kRing] = {};
    int pin_next = 0;
    // what the device holds: an unchanged set of bounds on the same stream is not uploaded again
    std::vector<float> eb_on_device;
    void* eb_stream = nullptr;
    // single-pass path: the device holds a codebook built from the previous call's payload under the current bounds
    bool carry_ready = false;
};

static size_t a256(size_t x) { return (x + 255) & ~size_t(255); }

static bool make_geom(const dlc_config* c, Geom* g) {
    if (!c) return false;
    if (c->dtype != DLC_F32 && c->dtype != DLC_F16) return false;
    if (c->num_tables < 1 || c->batch < 1 || c->dim < 1) return false;
    if (c->batch > 0x7FFFFFFFll || c->dim > 0x7FFFFFFFll) return false;
    const uint64_t n = (uint64_t)c->batch * (uint64_t)c->dim;
    if (n > 0x7FFFFFFFull) return false;
    const int R = c->radius;
    if (R < 8 || R > 2048 || (R & (R - 1))) return false;
    const int L = c->max_code_len;
    if (L < 1 || L > kLmaxLimit || (1 << L) < 2 * R) return false;
    const int S = c->chunk_symbols;
    if (S != 64 && S != 128 && S != 256) return false;
    if (c->flags & ~(int32_t)(DLC_FLAG_CARRY_CODEBOOK | DLC_FLAG_ROW_MATCH | DLC_FLAG_STATS_WORKSPACE | DLC_FLAG_SAMPLE_CODEBOOK)) return false;
    if ((c->flags & DLC_FLAG_SAMPLE_CODEBOOK) && (c->flags & DLC_FLAG_CARRY_CODEBOOK)) return false;  // one source of the codebook
    if (c->flags & DLC_FLAG_ROW_MATCH) {  // not with the other flags, and a lane's four elements must lie in one row
        if ((c->flags & ~(int32_t)DLC_FLAG_STATS_WORKSPACE) != DLC_FLAG_ROW_MATCH || c->dim % 4 != 0) return false;
    }
    const int64_t nd = c->num_dest == 0 ? 1 : c->num_dest;  // 0: a zero-initialised field means one destination
    if (nd < 1 || nd > 4096) return false;
    const uint64_t T = (uint64_t)c->num_tables * (uint64_t)nd;  // tables of the whole payload
    if (T > 0x7FFFFFFFull) return false;
    const uint64_t GS = (uint64_t)kW * S;
    const uint64_t G = (n + GS - 1) / GS;
    const uint64_t NG = G * T;
    if (NG * GS > 0xFFFFFFFFull) return false;                                 // element positions are 32-bit
    if (NG * kW * (((uint64_t)S * L + 31) / 32) > 0xFFFFFFFFull) return false;  // word offsets are 32-bit
    // ... also when every element of a container is an escape (two more words each): group offsets, scan records and
    // word ranges could not say where such a payload's groups start
    if ((uint64_t)c->num_tables * G * kW * (((uint64_t)S * L + 31) / 32) + 2ull * n * (uint64_t)c->num_tables > 0xFFFFFFFFull) return false;
    g->ND = (uint32_t)nd; g->TD = (uint32_t)c->num_tables;
    g->T = (uint32_t)T; g->B = (uint32_t)c->batch; g->D = (uint32_t)c->dim; g->n = (uint32_t)n;
    g->G = (uint32_t)G; g->NG = (uint32_t)NG; g->S = (uint32_t)S; g->R = (uint32_t)R; g->K = 2u * R;
    g->LMAX = (uint32_t)L; g->dtype = (uint32_t)c->dtype; g->es = c->dtype == DLC_F16 ? 2u : 4u;
    g->vec = (n % 4 == 0) ? 1u : 0u;
    g->lz = (c->flags & DLC_FLAG_ROW_MATCH) ? 1u : 0u;
    g->carry = (c->flags & DLC_FLAG_CARRY_CODEBOOK) ? 1u : 0u;
    g->sample = (c->flags & DLC_FLAG_SAMPLE_CODEBOOK) ? 1u : 0u;
    if (g->lz && T > 65535ull) return false;  // the row kernels' grids have a table per y index
    return true;
}

static size_t a16(size_t x) { return (x + 15) & ~size_t(15); }

extern "C" size_t dlc_compress_bound(const dlc_config* cfg) {
    Geom g;
    if (!make_geom(cfg, &g)) return 0;
    const FixedLayout F = fixed_layout(g);
    const size_t wpc = ((size_t)g.S * g.LMAX + 31) / 32;
    // one container: every chunk full, every element an escape, every symbol used
    const size_t off_cb = a16(F.off_payload + 4 * wpc * kW * g.TD * g.G + 8 * (size_t)g.n * g.TD);
    size_t one = off_cb + (size_t)g.TD * ((g.K + 3) & ~3u);
    if (g.lz) one = a16(one) + (size_t)g.TD * a16(4 * (size_t)g.B);  // the row references
    return g.ND == 1 ? one : (size_t)g.ND * a256(one);  // several: one every `capacity / num_dest` bytes, see dlc_compress
}

// carve the workspace; with base == nullptr only sizes are computed
static size_t carve(const Geom& g, uint8_t* base, Ws* w) {
    size_t off = 0;
    auto take = [&](size_t bytes) {
        uint8_t* p = base ? base + off : nullptr;
        off = a256(off + bytes);
        return p;
    };
    uint8_t* qp = take(sizeof(QParam) * g.T);
    uint8_t* hist = take((size_t)g.T * g.K * 4);
    uint8_t* hview = take((size_t)g.T * g.K * 4);
    uint8_t* ctrl = take(sizeof(Ctrl));
    uint8_t* tmeta = take(sizeof(TMeta) * g.T);
    uint8_t* enc = take(2 * (size_t)g.T * g.K);
    uint8_t* lens = take((size_t)g.T * g.K);
    uint8_t* state = take(8 * (size_t)g.NG);
    uint8_t* ws0 = take(4 * (size_t)g.T);
    uint8_t* ws1 = take(4 * (size_t)g.T);
    uint8_t* plane = g.sample ? nullptr : take((size_t)g.NG * kW * g.S);  // (with a sampled codebook every call is a single pass)
    uint8_t* escc = take(4 * (size_t)g.T);
    uint8_t* rm_on = g.lz ? take(g.T) : nullptr;
    uint8_t* rm_ref = g.lz ? take(4 * (size_t)g.T * g.B) : nullptr;
    uint8_t* rm_hash = g.lz ? take(8 * (size_t)g.T * g.B) : nullptr;
    uint8_t* rm_own = g.lz ? take(4 * (size_t)g.T * g.B) : nullptr;
    uint8_t* rm_mult = g.lz ? take(32 * (size_t)(g.D / 4u)) : nullptr;
    uint8_t* dtab = take(sizeof(DecTable) * g.T);
    const bool single = g.carry != 0 || g.sample != 0;  // the single-pass path's buffers
    uint8_t* gtot = single ? take(4 * (size_t)g.NG) : nullptr;
    uint8_t* enc2 = g.carry ? take(2 * (size_t)g.T * g.K) : nullptr;
    uint8_t* lens2 = g.carry ? take((size_t)g.T * g.K) : nullptr;
    uint8_t* tmeta2 = g.carry ? take(sizeof(TMeta) * g.T) : nullptr;
    uint8_t* bsum2 = single ? take(4 * (size_t)g.ND * sum_blocks_per_dest(g)) : nullptr;
    uint8_t* bsum = single ? take(4 * (size_t)g.ND * sum_blocks_per_dest(g)) : nullptr;
    uint8_t* desc = take(4 * (size_t)g.T);
    uint8_t* darr = take(4 * (size_t)g.T);
    // the slots come last: they are by far the largest part and the only one that dlc_create does not clear (everything
    // before them starts at zero: counters, flags, histograms)
    uint8_t* slots = single ? take(4 * (size_t)g.NG * (size_t)carry_slot_words(g)) : nullptr;
    if (w) {
        w->base = base; w->bytes = off;
        w->qp = (QParam*)qp;
        w->hist = (uint32_t*)hist; w->hist_view = (uint32_t*)hview; w->ctrl = (Ctrl*)ctrl;
        w->tmeta = (TMeta*)tmeta;
        w->enc = (uint16_t*)enc; w->lens = lens; w->state = (uint64_t*)state;
        w->word_start = (uint32_t*)ws0; w->word_end = (uint32_t*)ws1;
        w->sym_plane = plane;
        w->esc_count = (uint32_t*)escc;
        w->gtot = (uint32_t*)gtot; w->bsum = (uint32_t*)bsum; w->slots = (uint32_t*)slots;
        w->enc_next = (uint16_t*)enc2; w->lens_next = lens2; w->tmeta_next = (TMeta*)tmeta2; w->bsum_next = (uint32_t*)bsum2;
        w->dtab = (DecTable*)dtab; w->dec_esc = (uint32_t*)desc; w->dec_arrive = (uint32_t*)darr;
        w->rm_on = rm_on; w->rm_ref = (uint32_t*)rm_ref; w->rm_hash = (uint64_t*)rm_hash; w->rm_own = (uint32_t*)rm_own;
        w->rm_mult = (uint32_t*)rm_mult;
    }
    return off;
}

extern "C" size_t dlc_workspace_bytes(const dlc_config* cfg) {
    Geom g;
    if (!make_geom(cfg, &g)) return 0;
    return carve(g, nullptr, nullptr);
}

// the statistics reduction's own buffers: allocated by the first dlc_stats call, or by dlc_create when the
// configuration asks for them there (DLC_FLAG_STATS_WORKSPACE), so that a later call never allocates
static int stats_workspace(const Geom& g, Ws& w) {
    if (w.stats_base) return DLC_OK;
    size_t off = 0;
    auto take = [&](size_t b) { size_t o = off; off = a256(off + b); return o; };
    const size_t o_probe = take(sizeof(QParam) * g.T);
    const size_t o_own = take(2ull * g.T * g.B * 4);
    const size_t o_mult = take(16ull * g.D);
    const size_t o_hash = take(2ull * g.T * g.B * 8);
    const size_t o_mm = take(8ull * g.T);
    const size_t o_un = take(8ull * g.T);
    uint8_t* base = nullptr;
    if (hipMalloc((void**)&base, off) != hipSuccess) { (void)hipGetLastError(); return DLC_ENOMEM; }
    w.stats_base = base; w.stats_bytes = off;
    w.probe = (QParam*)(base + o_probe); w.st_own = (uint32_t*)(base + o_own); w.st_mult = (uint32_t*)(base + o_mult);
    w.rowhash = (uint64_t*)(base + o_hash); w.st_minmax = (uint32_t*)(base + o_mm); w.st_unique = (uint32_t*)(base + o_un);
    return DLC_OK;
}

extern "C" int dlc_create(dlc_ctx** out, const dlc_config* cfg) {
    if (!out) return DLC_EINVAL;
    *out = nullptr;
    Geom g;
    if (!make_geom(cfg, &g)) return DLC_EINVAL;
    dlc_ctx* c = new (std::nothrow) dlc_ctx();
    if (!c) return DLC_ENOMEM;
    c->cfg = *cfg;
    c->g = g;
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return DLC_EHIP; }
    const size_t bytes = carve(g, nullptr, nullptr);
    uint8_t* base = nullptr;
    if (hipMalloc((void**)&base, bytes) != hipSuccess) { (void)hipGetLastError(); delete c; return DLC_ENOMEM; }
    carve(g, base, &c->ws);
    // (the slots of the single-pass path are written before they are read: they need no clearing)
    const size_t clear_bytes = c->ws.slots ? (size_t)((uint8_t*)c->ws.slots - base) : bytes;
    if (hipMemset(base, 0, clear_bytes) != hipSuccess) { (void)hipFree(base); delete c; return DLC_EHIP; }
    c->ws.carry = (cfg->flags & DLC_FLAG_CARRY_CODEBOOK) ? 1u : 0u;
    c->ws.sample = (cfg->flags & DLC_FLAG_SAMPLE_CODEBOOK) ? 1u : 0u;
    if (g.lz && hipMemset(c->ws.rm_on, 1, g.T) != hipSuccess) { (void)hipFree(base); delete c; return DLC_EHIP; }  // all tables
    if (g.lz) {
        std::vector<uint32_t> mult(8 * (size_t)(g.D / 4u));
        row_match_multipliers(mult.data(), g.D / 4u);
        if (hipMemcpy(c->ws.rm_mult, mult.data(), 4 * mult.size(), hipMemcpyHostToDevice) != hipSuccess) { (void)hipFree(base); delete c; return DLC_EHIP; }
    }
    if (compress_set_attributes() != hipSuccess || decompress_set_attributes() != hipSuccess || row_match_set_attributes() != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(base);
        delete c;
        return DLC_EHIP;
    }
    if (hipHostMalloc((void**)&c->pin, sizeof(QParam) * g.T * dlc_ctx::kRing, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(base);
        delete c;
        return DLC_ENOMEM;
    }
    for (int i = 0; i < dlc_ctx::kRing; ++i)
        if (hipEventCreateWithFlags(&c->pin_ev[i], hipEventDisableTiming) != hipSuccess) {
            dlc_destroy(c);
            return DLC_EHIP;
        }
    if ((cfg->flags & DLC_FLAG_STATS_WORKSPACE) && g.ND == 1) {
        if (const int rc = stats_workspace(g, c->ws); rc != DLC_OK) {
            dlc_destroy(c);
            return rc;
        }
    }
    *out = c;
    return DLC_OK;
}

extern "C" void dlc_destroy(dlc_ctx* c) {
    if (!c) return;
    (void)hipDeviceSynchronize();
    for (auto& r : c->prof.recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (auto e : c->prof.pool) (void)hipEventDestroy(e);
    for (int i = 0; i < dlc_ctx::kRing; ++i)
        if (c->pin_ev[i]) (void)hipEventDestroy(c->pin_ev[i]);
    if (c->pin) (void)hipHostFree(c->pin);
    if (c->ws.base) (void)hipFree(c->ws.base);
    if (c->ws.stats_base) (void)hipFree(c->ws.stats_base);
    delete c;
}

static QParam make_qparam(float eb) {
    QParam q;
    q.eb = eb;
    q.ebx2 = eb * 2.0f;
    q.inv = (float)(1.0 / (double)q.ebx2);
    std::memcpy(&q.eb_bits, &eb, 4);
    return q;
}

static bool good_eb(float e) { return e > 0.0f && std::isfinite(e); }

// ---- Algorithm 1 -----------------------------------------------------------------------------------
static int classify(double eta, const dlc_controller_params* p) {
    if (eta > p->h_small) return DLC_CLASS_SMALL;
    if (eta < p->h_large) return DLC_CLASS_LARGE;
    return DLC_CLASS_MEDIUM;
}

static double iteration_multiplier(const dlc_controller_params* p, int64_t i) {
    if (p->decay_kind == DLC_DECAY_NONE || p->decay_len <= 0) return 1.0;
    const int64_t end = p->decay_start + p->decay_len;
    if (i >= end) return 1.0;
    if (p->decay_kind == DLC_DECAY_DROP || i < p->decay_start) return p->decay_mult0;
    if (p->decay_kind == DLC_DECAY_LINEAR)
        return p->decay_mult0 - (p->decay_mult0 - 1.0) * (double)(i - p->decay_start) / (double)p->decay_len;
    if (p->decay_kind == DLC_DECAY_LOG)
        return p->decay_mult0 -
               (p->decay_mult0 - 1.0) * (std::log(1.0 + (double)(i - p->decay_start)) / std::log(1.0 + (double)p->decay_len));
    const int64_t steps = p->decay_steps;
    if (steps < 1) return 1.0;
    int64_t s = ((i - p->decay_start) * steps) / p->decay_len;
    if (s >= steps) return 1.0;
    return p->decay_mult0 - (p->decay_mult0 - 1.0) * (double)s / (double)steps;
}

extern "C" int dlc_set_error_bounds(dlc_ctx* c, const dlc_table_stats* st, const dlc_controller_params* p,
                                    const int32_t* cls_override, int64_t iteration, float* eb, int32_t* cls_out,
                                    void* stream) {
    if (!c || !eb) return DLC_EINVAL;
    const uint32_t T = c->g.TD;  // a bound per table; the destinations share them
    if (st) {
        if (!p) return DLC_EINVAL;
        if (p->decay_kind < DLC_DECAY_NONE || p->decay_kind > DLC_DECAY_LOG || (p->mode != 0 && p->mode != 1))
            return DLC_EINVAL;
        const double mult = iteration_multiplier(p, iteration);
        for (uint32_t t = 0; t < T; ++t) {
            const double eta = ((double)st[t].n_unique_raw - (double)st[t].n_unique_quant) / (double)st[t].n_unique_raw;
            int cls = classify(eta, p);
            if (cls_override && cls_override[t] >= 0) cls = cls_override[t];
            if (cls < DLC_CLASS_SMALL || cls > DLC_CLASS_LARGE) return DLC_EINVAL;
            const double range = (double)st[t].max - (double)st[t].min;
            double e = p->mode == 1 ? p->global_eb * range : p->global_eb;
            if (cls == DLC_CLASS_LARGE) e = e * p->alpha;
            if (cls == DLC_CLASS_SMALL) e = e / p->beta;
            e = e * mult;
            if (p->eb_min > 0.0 && e < p->eb_min) e = p->eb_min;
            if (p->eb_max > 0.0 && e > p->eb_max) e = p->eb_max;
            if (p->rel_floor > 0.0) {
                const double f = p->rel_floor * range;
                if (e < f) e = f;
            }
            eb[t] = (float)e;
            if (cls_out) cls_out[t] = cls;
        }
    }
    for (uint32_t t = 0; t < T; ++t)
        if (!good_eb(eb[t])) return DLC_EINVAL;
    if (c->bounds_set && c->eb_stream == stream && c->eb_on_device.size() == T &&
        memcmp(c->eb_on_device.data(), eb, sizeof(float) * T) == 0)
        return DLC_OK;
    const int slot = c->pin_next;
    c->pin_next = (slot + 1) % dlc_ctx::kRing;
    if (c->pin_used[slot] && hipEventSynchronize(c->pin_ev[slot]) != hipSuccess) return DLC_EHIP;  // copy 16 calls ago
    QParam* h = c->pin + (size_t)slot * c->g.T;
    for (uint32_t d = 0; d < c->g.ND; ++d)
        for (uint32_t t = 0; t < T; ++t) h[(size_t)d * T + t] = make_qparam(eb[t]);
    if (hipMemcpyAsync(c->ws.qp, h, sizeof(QParam) * c->g.T, hipMemcpyHostToDevice, (hipStream_t)stream) != hipSuccess)
        return DLC_EHIP;
    if (hipEventRecord(c->pin_ev[slot], (hipStream_t)stream) != hipSuccess) return DLC_EHIP;
    c->pin_used[slot] = true;
    c->bounds_set = true;
    c->eb_on_device.assign(eb, eb + T);
    c->carry_ready = false;  // new bounds, new symbol distribution: the next call builds its own codebook
    c->eb_stream = stream;
    return DLC_OK;
}

static bool aligned16(const void* p) { return p && (((uintptr_t)p) & 15u) == 0; }

// clears 64-bit words on a stream (a kernel, not a memset: a caller may be capturing the stream into a graph)
__global__ __launch_bounds__(256) void k_zero_words(uint64_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256u + threadIdx.x; i < n; i += (size_t)gridDim.x * 256u) p[i] = 0ull;
}

extern "C" int dlc_compress(dlc_ctx* c, const void* d_payload, void* d_out, size_t cap, uint64_t* d_out_bytes,
                            void* stream) {
    if (!c || !aligned16(d_payload) || !aligned16(d_out) || !d_out_bytes || (((uintptr_t)d_out_bytes) & 7u))
        return DLC_EINVAL;
    if (!c->bounds_set) return DLC_ESTATE;
    if (c->g.ND > 1) cap = (cap / c->g.ND) & ~size_t(255);  // per destination: container d starts at d * cap
    if (cap < fixed_layout(c->g).off_payload) {  // the fixed-size sections must fit: nothing is written but the size, 0
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(256), 0, (hipStream_t)stream, d_out_bytes, (size_t)1);
        return hipGetLastError() == hipSuccess ? DLC_ECAPACITY : DLC_EHIP;
    }
    c->epoch += 1;
    if (c->epoch >= (1ull << 30)) {  // look-back records carry a 30-bit call counter
        const size_t n = c->g.NG;
        hipLaunchKernelGGL(k_zero_words, dim3((unsigned)std::min<size_t>((n + 255) / 256, 4096)), dim3(256), 0, (hipStream_t)stream,
                           c->ws.state, n);
        if (hipGetLastError() != hipSuccess) return DLC_EHIP;
        c->epoch = 1;
    }
    const bool was_single_pass = c->ws.sample != 0 || (c->ws.carry != 0 && c->carry_ready);
    hipError_t e = launch_compress(c->g, d_payload, (uint8_t*)d_out, cap, d_out_bytes, c->ws, c->epoch, c->carry_ready,
                                   c->prof.level, &c->prof, (hipStream_t)stream);
    c->carry_ready = e == hipSuccess && c->ws.carry != 0;
    if (c->ws.carry != 0) {  // the codebook just built for the next call becomes the current one
        std::swap(c->ws.enc, c->ws.enc_next);
        std::swap(c->ws.lens, c->ws.lens_next);
        std::swap(c->ws.tmeta, c->ws.tmeta_next);
    }
    if (was_single_pass) std::swap(c->ws.bsum, c->ws.bsum_next);  // (the single-pass step has cleared the other set)
    return e == hipSuccess ? DLC_OK : DLC_EHIP;
}

extern "C" int dlc_decompress(dlc_ctx* c, const void* d_comp, size_t comp_bytes, void* d_out, size_t cap, void* stream) {
    if (!c || !aligned16(d_comp) || !aligned16(d_out)) return DLC_EINVAL;
    if (cap < (size_t)c->g.n * c->g.T * c->g.es) return DLC_ECAPACITY;
    if (c->g.ND > 1) comp_bytes = (comp_bytes / c->g.ND) & ~size_t(255);  // per container: container d starts at d * comp_bytes
    // the sections whose size the geometry fixes (header, directory, group and chunk tables) must be there
    if (comp_bytes < fixed_layout(c->g).off_payload) return DLC_ECORRUPT;
    hipError_t e = launch_decompress(c->g, (const uint8_t*)d_comp, comp_bytes, d_out, c->ws, c->prof.level, &c->prof,
                                     (hipStream_t)stream);
    return e == hipSuccess ? DLC_OK : DLC_EHIP;
}

// ---- decompression for callers that cannot allocate --------------------------------------------------------------
// The decode kernels' workspace (status word, per-table escape and arrival counters, the row references' table) is
// this array, part of the library's image on every GPU it is loaded on; the kernels get its address on the current
// device, looked up once per device, never the array's name.
constexpr uint32_t kStaticTables = DLC_STATIC_MAX_TABLES;
constexpr size_t kStaticCtrlBytes = 256;
constexpr size_t kStaticBytes = kStaticCtrlBytes + (size_t)kStaticTables * (4 + 4 + sizeof(DecTable));
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kStaticDevices = 64;
static std::mutex g_static_mu;
static unsigned char* g_static_ptr[kStaticDevices] = {};

static int static_scratch(unsigned char** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return DLC_EHIP;
    if (dev < 0 || dev >= kStaticDevices) return DLC_ELIMIT;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DLC_EHIP;
        if (decompress_set_attributes() != hipSuccess) return DLC_EHIP;
        g_static_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_static_ptr[dev];
    return DLC_OK;
}

// what must start at zero: the status word and the counters of the call's tables (a call that found a bad container
// may have left counters behind)
__global__ __launch_bounds__(256) void k_static_clear(uint32_t* ctrl_words, uint32_t* esc, uint32_t* arrive, uint32_t T) {
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i < sizeof(Ctrl) / 4u) ctrl_words[i] = 0u;
    if (i < T) esc[i] = arrive[i] = 0u;
}

__global__ void k_static_status(const Ctrl* ctrl, int32_t* status_out) { status_out[0] = ctrl->status; }

extern "C" int dlc_decompress_static(const dlc_config* cfg, const void* d_comp, size_t comp_bytes, void* d_out, size_t cap,
                                     int32_t* d_status, void* stream) {
    Geom g;
    if (!make_geom(cfg, &g) || !d_status || !aligned16(d_comp) || !aligned16(d_out)) return DLC_EINVAL;
    if (g.T > kStaticTables) return DLC_ELIMIT;
    if (cap < (size_t)g.n * g.T * g.es) return DLC_ECAPACITY;
    if (g.ND > 1) comp_bytes = (comp_bytes / g.ND) & ~size_t(255);
    if (comp_bytes < fixed_layout(g).off_payload) return DLC_ECORRUPT;
    unsigned char* base = nullptr;
    const int rc = static_scratch(&base);
    if (rc != DLC_OK) return rc;
    Ws w;
    w.ctrl = reinterpret_cast<Ctrl*>(base);
    w.dec_esc = reinterpret_cast<uint32_t*>(base + kStaticCtrlBytes);
    w.dec_arrive = w.dec_esc + kStaticTables;
    w.dtab = reinterpret_cast<DecTable*>(base + kStaticCtrlBytes + (size_t)kStaticTables * 8);
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_static_clear, dim3((std::max<uint32_t>(g.T, 8u) + 255u) / 256u), dim3(256), 0, s,
                       reinterpret_cast<uint32_t*>(base), w.dec_esc, w.dec_arrive, g.T);
    hipError_t e = launch_decompress(g, (const uint8_t*)d_comp, comp_bytes, d_out, w, 0, nullptr, s);
    hipLaunchKernelGGL(k_static_status, dim3(1), dim3(1), 0, s, w.ctrl, d_status);
    if (e == hipSuccess) e = hipGetLastError();
    return e == hipSuccess ? DLC_OK : DLC_EHIP;
}

extern "C" int dlc_set_row_match(dlc_ctx* c, const uint8_t* h_flags, void* stream) {
    if (!c) return DLC_EINVAL;
    if (!c->g.lz) return DLC_ESTATE;
    std::vector<uint8_t> f(c->g.T, 1);
    if (h_flags)
        for (uint32_t t = 0; t < c->g.T; ++t) f[t] = h_flags[t % c->g.TD] ? 1 : 0;  // the same for every destination
    if (hipMemcpyAsync(c->ws.rm_on, f.data(), c->g.T, hipMemcpyHostToDevice, (hipStream_t)stream) != hipSuccess) return DLC_EHIP;
    return hipStreamSynchronize((hipStream_t)stream) == hipSuccess ? DLC_OK : DLC_EHIP;  // f goes out of scope
}

extern "C" int dlc_read_row_refs(dlc_ctx* c, uint32_t* h_ref, void* stream) {
    if (!c || !h_ref) return DLC_EINVAL;
    if (!c->g.lz) return DLC_ESTATE;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return DLC_EHIP;
    return hipMemcpy(h_ref, c->ws.rm_ref, 4ull * c->g.T * c->g.B, hipMemcpyDeviceToHost) == hipSuccess ? DLC_OK : DLC_EHIP;
}

extern "C" int dlc_set_row_hash_multipliers(dlc_ctx* c, const uint32_t* h_mult, void* stream) {
    if (!c || !h_mult) return DLC_EINVAL;
    if (!c->g.lz) return DLC_ESTATE;
    if (hipMemcpyAsync(c->ws.rm_mult, h_mult, 32 * (size_t)(c->g.D / 4u), hipMemcpyHostToDevice, (hipStream_t)stream) != hipSuccess) return DLC_EHIP;
    return hipStreamSynchronize((hipStream_t)stream) == hipSuccess ? DLC_OK : DLC_EHIP;
}

extern "C" double dlc_speedup_estimate(double cr, double net_gbps, double tc_gbps, double td_gbps) {
    if (!(cr > 0.0) || !(net_gbps > 0.0) || !(tc_gbps > 0.0) || !(td_gbps > 0.0)) return 0.0;
    return 1.0 / (1.0 / cr + net_gbps * (1.0 / tc_gbps + 1.0 / td_gbps));
}

// The offline procedure of the algorithm "Compressor Selection" (Section III-D) for the two compressors of this library.
extern "C" int dlc_select_compressors(dlc_ctx* c, const void* d_sample, void* d_out, size_t out_capacity, uint64_t* d_out_bytes,
                                      void* d_rec, size_t rec_capacity, double net_gbps, const double* h_tc_gbps,
                                      const double* h_td_gbps, uint8_t* h_choice_out, double* h_speedup_out, void* stream) {
    if (!c || !h_choice_out || !(net_gbps > 0.0)) return DLC_EINVAL;
    if ((h_tc_gbps == nullptr) != (h_td_gbps == nullptr)) return DLC_EINVAL;
    if (!c->g.lz || c->g.ND != 1) return DLC_ESTATE;  // needs both compressors, and one container
    const bool measure = h_tc_gbps == nullptr;
    if (measure && !d_rec) return DLC_EINVAL;
    const uint32_t T = c->g.T;
    hipStream_t s = (hipStream_t)stream;
    const double raw_table = (double)c->g.n * c->g.es, raw_all = raw_table * T;
    std::vector<uint64_t> sizes[2];
    double tc[2], td[2];
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (measure && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) {
        if (e0) (void)hipEventDestroy(e0);
        return DLC_EHIP;
    }
    int rc = DLC_OK;
    std::vector<uint8_t> flags(T);
    for (int comp = 0; comp < 2 && rc == DLC_OK; ++comp) {
        std::fill(flags.begin(), flags.end(), (uint8_t)comp);
        rc = dlc_set_row_match(c, flags.data(), stream);
        if (rc == DLC_OK) rc = dlc_compress(c, d_sample, d_out, out_capacity, d_out_bytes, stream);
        if (rc == DLC_OK) rc = dlc_sync_status(c, stream);
        if (rc != DLC_OK) break;
        sizes[comp].resize(1 + (size_t)T);
        if (hipMemcpy(sizes[comp].data(), d_out_bytes, 8 * (1 + (size_t)T), hipMemcpyDeviceToHost) != hipSuccess) { rc = DLC_EHIP; break; }
        if (measure) {  // the rates of this compressor on the sample: a few calls between two events, each direction
            const int reps = 3;
            float ms = 0.f;
            if (hipEventRecord(e0, s) != hipSuccess) { rc = DLC_EHIP; break; }
            for (int i = 0; i < reps && rc == DLC_OK; ++i) rc = dlc_compress(c, d_sample, d_out, out_capacity, d_out_bytes, stream);
            if (rc != DLC_OK) break;
            if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { rc = DLC_EHIP; break; }
            tc[comp] = raw_all * reps / ((double)ms * 1e6);
            if (hipEventRecord(e0, s) != hipSuccess) { rc = DLC_EHIP; break; }
            for (int i = 0; i < reps && rc == DLC_OK; ++i) rc = dlc_decompress(c, d_out, (size_t)sizes[comp][0], d_rec, rec_capacity, stream);
            if (rc != DLC_OK) break;
            if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { rc = DLC_EHIP; break; }
            td[comp] = raw_all * reps / ((double)ms * 1e6);
            rc = dlc_sync_status(c, stream);
        } else {
            tc[comp] = h_tc_gbps[comp];
            td[comp] = h_td_gbps[comp];
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (rc != DLC_OK) return rc;
    for (uint32_t t = 0; t < T; ++t) {
        // per table the compressor with the larger estimate; the entropy coder alone (listed first) when they are equal
        const double s0 = dlc_speedup_estimate(raw_table / (double)sizes[0][1 + t], net_gbps, tc[0], td[0]);
        const double s1 = dlc_speedup_estimate(raw_table / (double)sizes[1][1 + t], net_gbps, tc[1], td[1]);
        flags[t] = s1 > s0 ? 1 : 0;
        h_choice_out[t] = flags[t];
        if (h_speedup_out) h_speedup_out[t] = s1 > s0 ? s1 : s0;
    }
    return dlc_set_row_match(c, flags.data(), stream);
}

extern "C" int dlc_sync_status(dlc_ctx* c, void* stream) {
    if (!c) return DLC_EINVAL;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return DLC_EHIP;
    int32_t st = 0;
    if (hipMemcpy(&st, &c->ws.ctrl->status, 4, hipMemcpyDeviceToHost) != hipSuccess) return DLC_EHIP;
    if (st != 0) {
        if (hipMemset(&c->ws.ctrl->status, 0, 4) != hipSuccess) return DLC_EHIP;
    }
    return st;
}

static float ord_dec(uint32_t o) {
    uint32_t b = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
    float f;
    std::memcpy(&f, &b, 4);
    return f;
}

extern "C" int dlc_stats(dlc_ctx* c, const void* d_payload, const float* probe_eb, dlc_table_stats* out, void* stream) {
    if (!c || !aligned16(d_payload) || !probe_eb || !out) return DLC_EINVAL;
    const Geom& g = c->g;
    if (g.ND != 1) return DLC_ESTATE;  // a table's statistics are over its whole batch: use a context that is not split
    if (g.T > 65535u) return DLC_EINVAL;  // the kernels' grids have a table per y index
    for (uint32_t t = 0; t < g.T; ++t)
        if (!good_eb(probe_eb[t])) return DLC_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    Ws& w = c->ws;
    if (const int rc = stats_workspace(g, w); rc != DLC_OK) return rc;
    std::vector<QParam> pq(g.T);
    for (uint32_t t = 0; t < g.T; ++t) pq[t] = make_qparam(probe_eb[t]);
    std::vector<uint32_t> mm(2 * g.T), un(2 * g.T);
    if (hipMemcpyAsync(w.probe, pq.data(), sizeof(QParam) * g.T, hipMemcpyHostToDevice, s) != hipSuccess) return DLC_EHIP;
    for (uint32_t attempt = 0; attempt < 4; ++attempt) {
        // (the first kernel of the reduction clears the range words, the counts and the collision counter)
        if (launch_stats(g, d_payload, w.probe, w, 0x51ED270Bu * (attempt + 1), s) != hipSuccess) return DLC_EHIP;
        uint32_t collide = 0;
        int32_t st = 0;
        if (hipMemcpyAsync(mm.data(), w.st_minmax, 8ull * g.T, hipMemcpyDeviceToHost, s) != hipSuccess) return DLC_EHIP;
        if (hipMemcpyAsync(un.data(), w.st_unique, 8ull * g.T, hipMemcpyDeviceToHost, s) != hipSuccess) return DLC_EHIP;
        if (hipMemcpyAsync(&collide, &w.ctrl->collide, 4, hipMemcpyDeviceToHost, s) != hipSuccess) return DLC_EHIP;
        if (hipMemcpyAsync(&st, &w.ctrl->status, 4, hipMemcpyDeviceToHost, s) != hipSuccess) return DLC_EHIP;
        if (hipStreamSynchronize(s) != hipSuccess) return DLC_EHIP;
        if (st != DLC_OK) {
            if (hipMemset(&w.ctrl->status, 0, 4) != hipSuccess) return DLC_EHIP;
            return st;
        }
        if (collide == 0) {
            for (uint32_t t = 0; t < g.T; ++t) {
                out[t].min = mm[2 * t] == 0xFFFFFFFFu ? std::numeric_limits<float>::infinity() : ord_dec(mm[2 * t]);
                out[t].max = mm[2 * t + 1] == 0u ? -std::numeric_limits<float>::infinity() : ord_dec(mm[2 * t + 1]);
                out[t].count = g.n;
                out[t].n_rows = g.B;
                out[t].n_unique_raw = un[2 * t];
                out[t].n_unique_quant = un[2 * t + 1];
                out[t].probe_eb = probe_eb[t];
            }
            return DLC_OK;
        }
    }
    return DLC_ESTATE;  // four different hash salts all collided: not expected
}

extern "C" int dlc_quantize(dlc_ctx* c, const void* d_payload, uint16_t* d_sym, void* stream) {
    if (!c || !aligned16(d_payload) || !d_sym) return DLC_EINVAL;
    if (!c->bounds_set) return DLC_ESTATE;
    if (launch_quantize(c->g, d_payload, c->ws.qp, d_sym, (hipStream_t)stream) != hipSuccess) return DLC_EHIP;
    return hipStreamSynchronize((hipStream_t)stream) == hipSuccess ? DLC_OK : DLC_EHIP;
}

extern "C" int dlc_read_histogram(dlc_ctx* c, uint32_t* h_hist, void* stream) {
    if (!c || !h_hist) return DLC_EINVAL;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return DLC_EHIP;
    return hipMemcpy(h_hist, c->ws.hist_view, 4ull * c->g.T * c->g.K, hipMemcpyDeviceToHost) == hipSuccess ? DLC_OK
                                                                                                            : DLC_EHIP;
}

extern "C" int dlc_read_codebook(dlc_ctx* c, uint8_t* h_len, uint16_t* h_code, void* stream) {
    if (!c || !h_len || !h_code) return DLC_EINVAL;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return DLC_EHIP;
    const size_t n = (size_t)c->g.T * c->g.K;
    if (hipMemcpy(h_len, c->ws.lens, n, hipMemcpyDeviceToHost) != hipSuccess) return DLC_EHIP;
    if (hipMemcpy(h_code, c->ws.enc, 2 * n, hipMemcpyDeviceToHost) != hipSuccess) return DLC_EHIP;
    for (size_t i = 0; i < n; ++i) h_code[i] &= 0x0FFFu;
    return DLC_OK;
}

extern "C" int dlc_profile_enable(dlc_ctx* c, int level) {
    if (!c || level < 0 || level > 2) return DLC_EINVAL;
    c->prof.level = level;
    return DLC_OK;
}

extern "C" int dlc_profile_read(dlc_ctx* c, int max_slots, const char** names, float* total_ms, int32_t* launches) {
    if (!c) return DLC_EINVAL;
    Prof& p = c->prof;
    for (auto& r : p.recs) {
        if (hipEventSynchronize(r.b) != hipSuccess) return DLC_EHIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) { p.total_ms[r.slot] += ms; p.launches[r.slot] += 1; }
        p.pool.push_back(r.a);
        p.pool.push_back(r.b);
    }
    p.recs.clear();
    for (int i = 0; i < P_NSLOTS && i < max_slots; ++i) {
        if (names) names[i] = kSlotNames[i];
        if (total_ms) total_ms[i] = p.total_ms[i];
        if (launches) launches[i] = p.launches[i];
    }
    for (int i = 0; i < P_NSLOTS; ++i) { p.total_ms[i] = 0.f; p.launches[i] = 0; }
    return P_NSLOTS;
}

extern "C" const char* dlc_strerror(int s) {
    switch (s) {
        case DLC_OK: return "ok";
        case DLC_EINVAL: return "invalid argument";
        case DLC_ENOMEM: return "out of device memory";
        case DLC_ECAPACITY: return "output capacity too small";
        case DLC_ECORRUPT: return "corrupt or mismatching container";
        case DLC_EHIP: return "HIP runtime error";
        case DLC_ESTATE: return "bad call order or internal invariant";
        case DLC_ELIMIT: return "beyond the fixed maximum of an entry point that allocates nothing";
        default: return "unknown status";
    }
}
