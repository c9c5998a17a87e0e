// Host side of libfluxmoe.so: context, offline encode driver, tier binding, the
// materialize / expert-FFN enqueue paths and the event protocol between them.
//
// Event protocol = PagedTensor synchronization (paper Alg. 1), generalised from the two
// reusable layer blocks to individual staging slots: a materialize waits for the inference
// event of every layer whose FFN last read one of its target slots (write-after-read); an
// FFN call waits for its layer's load event (read-after-write) and records the layer's
// inference event.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <atomic>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <new>
#include <thread>

#include "fluxmoe_internal.h"

namespace fluxmoe {

static thread_local char g_err[512] = "";

int set_error(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}

}  // namespace fluxmoe

using namespace fluxmoe;

#define HIPCHECK(call)                                                                  \
    do {                                                                                \
        hipError_t e_ = (call);                                                         \
        if (e_ != hipSuccess)                                                           \
            return set_error(FLUXMOE_EHIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

namespace {
constexpr int kRing = 4;
constexpr uint32_t kLutBytes = kLutEntries * 4;

// What one half of the host-tier staging buffer currently holds.
struct StageHalf {
    int64_t layer = -1;            // layer whose host-tier blocks are staged, -1 = nothing
    std::vector<int64_t> off[2];   // per expert: byte offset of the tensor's host part, -1 = absent
};

struct FfnPlan {
    uint32_t m_tile, ksplit, pairs_cap, tiles_cap, n_chunks;
    uint64_t bytes;
    uint64_t off_count, off_offset, off_sorted, off_pos, off_tile, off_ntiles, off_chunk, off_h, off_y;
};

inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }
}  // namespace

// FFN scratch of fluxmoe_expert_ffn_static: one array per GPU, part of the loaded code object, held until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the device
// address of each GPU's copy is resolved once per device (resolve_static_scratch, called by
// fluxmoe_bind_arenas with that device current) and kept in g_static_scratch.
constexpr uint64_t kStaticScratchBytes = FLUXMOE_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];
static uint8_t* g_static_scratch[kMaxDevices] = {};

struct fluxmoe_ctx {
    fluxmoe_desc d;
    int device = -1;                      // HIP device the arenas were bound on
    uint64_t elems13 = 0, elems2 = 0;
    std::vector<LayerMeta> layers;
    // arenas
    uint8_t* slots13 = nullptr;
    uint8_t* slots2 = nullptr;
    uint8_t* ws = nullptr;
    size_t ws_bytes = 0;
    bool arenas_bound = false;
    int n_cus = 256;
    // pool workspace layout
    uint64_t lut_off = 0, cmd_off = 0, err_off = 0, pool_ws_bytes = 0;
    uint32_t max_jobs = 0, max_upd = 0, cmd_bytes = 0;
    // command ring (pinned host mirror of the device command buffers)
    uint8_t* pinned_cmd = nullptr;
    hipEvent_t ring_ev[kRing] = {};
    bool ring_used[kRing] = {};
    int ring_next = 0;
    // page-table mirror and slot ownership
    std::vector<int32_t> pt;
    std::vector<int64_t> slot_owner;      // layer * E + expert, or -1
    // Alg. 1 state
    std::vector<hipEvent_t> ev_load, ev_infer, ev_rel;   // per layer: last materialize / FFN / release
    std::vector<uint8_t> load_valid, infer_valid, rel_valid;
    std::vector<int32_t> slot_last_reader; // layer whose FFN last read the slot, or -1
    bool events_ready = false;
    // host-tier staging
    uint8_t* staging = nullptr;
    size_t staging_bytes = 0;
    StageHalf half[2];                      // layer l stages into half l & 1
    hipEvent_t ev_copied[2] = {};           // copies into the half have completed
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;   // fluxmoe_materialize_two_streams
    hipEvent_t ev_half_done[2] = {};        // last decode that read the half
    bool half_done_valid[2] = {false, false};
    bool copied_valid[2] = {false, false};  // ev_copied[h] has been recorded
    // launch shape of the decode kernel (FLUXMOE_DECODE_WAVES / FLUXMOE_DECODE_BLOCKS_PER_WAVE override)
    int tune_waves = 8;
    int tune_blocks_per_wave = 3;
    int tune_tiled_waves = 2;             // FLUXMOE_FFN_TILED_WAVES: 2 = LDS-direct loads (default), 8 = register-staged,
                                          // 4 = register-staged with four wavefronts of 128 x 128
    int tune_tiled_persist = 1;           // FLUXMOE_FFN_TILED_PERSIST: 0 = one workgroup per tile, n = n x 256 workgroups walking the tiles
    int tune_tiled_group = 0;             // FLUXMOE_FFN_TILED_GROUP: 1..8 super-rows per group of the tiled gate/up kernel, 0 = from the shape
    // optional kernel timing (fluxmoe_profile_*)
    bool profiling = false;
    uint32_t profile_mask = 0x1F;         // kinds that are bracketed while profiling
    bool span_open = false;               // the span begun last is being recorded
    struct Span { hipEvent_t a, b; int kind; };
    std::vector<Span> spans;
};

namespace {

void compute_layout(fluxmoe_ctx* c) {
    const uint64_t E = c->d.n_experts;
    c->max_jobs = uint32_t(2 * E + 2);
    c->max_upd = uint32_t(2 * E + 2);
    c->cmd_bytes = uint32_t(align_up(sizeof(DecodeCmd) + 2ull * c->max_jobs * sizeof(DecodeJob) +
                                     c->max_upd * 8ull, 256));
    c->lut_off = 0;
    c->cmd_off = align_up(uint64_t(c->d.n_layers) * 2 * kLutBytes, 256);
    c->err_off = c->cmd_off + uint64_t(kRing) * c->cmd_bytes;
    c->pool_ws_bytes = align_up(c->err_off + 256, 4096);
}

// Shapes and launch parameters the FFN plan depends on (a routed layer, or one always-mapped expert
// for the shared-expert call).
struct FfnShape {
    uint64_t E, H, F;
    int n_cus, tiled_waves;
};

FfnShape ffn_shape(const fluxmoe_ctx* c, uint32_t n_experts) {
    return FfnShape{n_experts, c->d.hidden, c->d.ffn, c->n_cus, c->tune_tiled_waves};
}

FfnPlan plan_ffn(const FfnShape& c, uint32_t T, uint32_t K) {
    FfnPlan p{};
    const uint64_t E = c.E, H = c.H, F = c.F;
    const uint64_t pairs = uint64_t(T) * K;
    const uint64_t groups = std::max<uint64_t>(1, std::min<uint64_t>(E, pairs));
    const uint64_t avg = (pairs + groups - 1) / groups;
    // Row tile of the weight-streaming kernels: every extra tile of an expert streams that expert's
    // weights again, and routing can be far from even, so tiles hold up to 128 rows (the kernel takes a
    // cheaper body for tiles with fewer rows).  With so many rows per expert that even 128-row tiles are
    // exceeded often (an expert's row count taken as normal with mean and variance avg), 128-row tiles
    // stay the choice while the expected number of passes per expert is below 1.6 - what one pass of
    // the LDS-tiled MFMA kernels (256-row tiles, k extents that are multiples of 64) costs relative to
    // a streaming pass at these sizes.
    auto p_over = [&](double m) { return 0.5 * std::erfc((m + 0.5 - double(avg)) / std::sqrt(2.0 * double(avg))); };
    p.m_tile = 128;
    if (p_over(128) > 0.02 && 1.0 + p_over(128) + p_over(256) + p_over(384) > 1.6 && H % 64 == 0 && F % 64 == 0)
        p.m_tile = 256;
    if (const char* v = std::getenv("FLUXMOE_FFN_MTILE")) {
        const int m = std::atoi(v);
        if (m == 16 || m == 32 || m == 64 || m == 96 || m == 128 || (m == 256 && H % 64 == 0 && F % 64 == 0)) p.m_tile = uint32_t(m);
    }
    p.pairs_cap = uint32_t(std::max<uint64_t>(pairs, 1));
    p.tiles_cap = uint32_t(pairs / p.m_tile + groups + 1);
    // Split K of the second product (strip kernels).  One workgroup (four strips, one per SIMD) fits on a
    // CU at a time, so the launch runs in rounds of n_cus workgroups; the split is the one with the
    // smallest estimated time in units of k rows per workgroup: rounds x (rows per split + a fixed
    // start-up cost) + the FP32 partials it writes and combine_kernel reads back.
    const uint64_t strips2 = (H + 127) / 128;
    const uint64_t est_tiles = std::max<uint64_t>(1, std::max<uint64_t>(pairs / p.m_tile, std::min(groups, pairs)));
    const uint64_t n_cus = uint64_t(std::max(c.n_cus, 1));
    uint64_t ks = 1, best_cost = ~0ull;
    for (uint64_t k = 1; k <= 8 && k <= std::max<uint64_t>(1, F / 256); ++k) {
        const uint64_t wgs = (strips2 + 3) / 4 * est_tiles * k;
        const uint64_t rounds = (wgs + n_cus - 1) / n_cus;
        const uint64_t partials = k > 1 ? k * pairs * H * 8 / (n_cus * 1024) : 0;
        const uint64_t cost = rounds * ((F + k - 1) / k + 384) + partials;
        if (cost < best_cost) { best_cost = cost; ks = k; }
    }
    p.ksplit = uint32_t(ks);
    if (p.m_tile == 256) {
        // LDS-tiled kernels: one 256 x 256 tile per workgroup.  When the second product has fewer tiles
        // than the chip has CUs, the LDS-direct kernel splits K so that about one workgroup per CU runs
        // (each split keeps at least 8 steps of 64)
        p.ksplit = 1;
        if (c.tiled_waves == 2 || c.tiled_waves == 1) {
            const uint64_t tiles2 = groups * ((avg + 255) / 256) * ((H + 255) / 256);
            uint64_t k2 = std::max<uint64_t>(1, n_cus / tiles2);
            k2 = std::min<uint64_t>(k2, 8);
            k2 = std::min<uint64_t>(k2, std::max<uint64_t>(1, F / 512));
            p.ksplit = uint32_t(k2);
        }
    }
    uint64_t o = 0;
    auto take = [&](uint64_t bytes) { uint64_t at = o; o = align_up(o + bytes, 256); return at; };
    p.off_count = take((E + 1) * 4);
    p.off_offset = take((E + 2) * 4);
    p.off_sorted = take(uint64_t(p.pairs_cap) * 4);
    p.off_pos = take(uint64_t(p.pairs_cap) * 4);
    p.off_tile = take(uint64_t(p.tiles_cap) * 16);
    p.off_ntiles = take(4);
    p.n_chunks = pairs > kRouteChunkThreshold ? uint32_t((pairs + kRouteChunkPairs - 1) / kRouteChunkPairs) : 0u;
    p.off_chunk = take(uint64_t(p.n_chunks) * E * 4);
    p.off_h = take(uint64_t(p.pairs_cap) * F * 2);
    p.off_y = take(uint64_t(p.ksplit) * p.pairs_cap * H * 4);
    p.bytes = o;
    return p;
}

// Pair table of the decode kernel, indexed by the next 12 stream bits (first stream bit in bit 0).
// Entry: bits 0..5 bits to advance, 7..14 first exponent, 15..18 length of the first code, 23..30
// second exponent, bit 31 set when the second code does not end inside the 12 bits (the entry then
// covers the first symbol only).  Bit patterns no code matches (only possible with a single used
// symbol) decode as the first used symbol with length 1: valid streams never reach them.
void build_lut(const uint8_t lens[256], uint32_t* lut) {
    uint16_t codes[256];
    canonical_codes(lens, codes);
    int fallback = -1;
    for (int s = 0; s < 256; ++s)
        if (lens[s]) { fallback = s; break; }
    // single-symbol table: 12 stream bits -> (symbol, length)
    std::vector<uint16_t> one(kLutEntries, uint16_t(fallback < 0 ? 1 : ((fallback << 4) | 1)));
    for (int s = 0; s < 256; ++s) {
        const uint32_t L = lens[s];
        if (!L || L > kLutBits) continue;
        uint32_t rev = 0;   // first code bit in bit 0: that is how the stream is peeked
        for (uint32_t b = 0; b < L; ++b) rev |= ((codes[s] >> (L - 1 - b)) & 1u) << b;
        for (uint32_t hi = 0; hi < (1u << (kLutBits - L)); ++hi)
            one[rev | (hi << L)] = uint16_t((s << 4) | L);
    }
    for (uint32_t i = 0; i < kLutEntries; ++i) {
        const uint32_t s0 = one[i] >> 4, l0 = one[i] & 15u;
        uint32_t entry = 0x80000000u | (l0 << 15) | (s0 << 7) | l0;
        if (l0 < kLutBits) {
            // the second code must end inside the remaining 12 - l0 bits; the bits above them are zero
            // in this index, so a match longer than what remains is not a match
            const uint32_t rest = i >> l0;
            const uint32_t s1 = one[rest] >> 4, l1 = one[rest] & 15u;
            bool real = false;                      // is `rest` really the code of s1, not the fallback?
            if (lens[s1] == l1) {
                uint32_t rev = 0;
                for (uint32_t b = 0; b < l1; ++b) rev |= ((codes[s1] >> (l1 - 1 - b)) & 1u) << b;
                real = (rest & ((1u << l1) - 1u)) == rev;
            }
            if (real && l0 + l1 <= kLutBits) entry = (s1 << 23) | (l0 << 15) | (s0 << 7) | (l0 + l1);
        }
        lut[i] = entry;
    }
}

int check_layer(const fluxmoe_ctx* c, uint32_t layer, bool need_encoded) {
    if (!c) return set_error(FLUXMOE_EINVAL, "ctx is NULL");
    if (layer >= c->d.n_layers)
        return set_error(FLUXMOE_ERANGE, "layer %u out of range (n_layers %u)", layer, c->d.n_layers);
    if (need_encoded && !c->layers[layer].encoded)
        return set_error(FLUXMOE_ESTATE, "layer %u has not been encoded", layer);
    return FLUXMOE_OK;
}

int ensure_events(fluxmoe_ctx* c) {
    if (c->events_ready) return FLUXMOE_OK;
    const uint32_t N = c->d.n_layers;
    c->ev_load.assign(N, nullptr);
    c->ev_infer.assign(N, nullptr);
    c->ev_rel.assign(N, nullptr);
    for (uint32_t i = 0; i < N; ++i) {
        HIPCHECK(hipEventCreateWithFlags(&c->ev_load[i], hipEventDisableTiming));
        HIPCHECK(hipEventCreateWithFlags(&c->ev_infer[i], hipEventDisableTiming));
        HIPCHECK(hipEventCreateWithFlags(&c->ev_rel[i], hipEventDisableTiming));
    }
    for (int i = 0; i < kRing; ++i)
        HIPCHECK(hipEventCreateWithFlags(&c->ring_ev[i], hipEventDisableTiming));
    HIPCHECK(hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming));
    HIPCHECK(hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming));
    for (int i = 0; i < 2; ++i) {
        HIPCHECK(hipEventCreateWithFlags(&c->ev_half_done[i], hipEventDisableTiming));
        HIPCHECK(hipEventCreateWithFlags(&c->ev_copied[i], hipEventDisableTiming));
    }
    HIPCHECK(hipHostMalloc(reinterpret_cast<void**>(&c->pinned_cmd), size_t(kRing) * c->cmd_bytes,
                           hipHostMallocDefault));
    c->events_ready = true;
    return FLUXMOE_OK;
}

int resolve_static_scratch(int dev) {
    if (dev < 0 || dev >= kMaxDevices) return set_error(FLUXMOE_EHIP, "device index %d out of range", dev);
    if (g_static_scratch[dev]) return FLUXMOE_OK;
    void* ptr = nullptr;
    HIPCHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return set_error(FLUXMOE_EHIP, "hipGetSymbolAddress returned a NULL address");
    g_static_scratch[dev] = static_cast<uint8_t*>(ptr);
    return FLUXMOE_OK;
}

hipError_t span_begin(fluxmoe_ctx* c, int kind, hipStream_t s) {
    c->span_open = c->profiling && ((c->profile_mask >> kind) & 1u);
    if (!c->span_open) return hipSuccess;
    fluxmoe_ctx::Span sp{nullptr, nullptr, kind};
    hipError_t e = hipEventCreate(&sp.a);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&sp.b);
    if (e != hipSuccess) return e;
    c->spans.push_back(sp);
    return hipEventRecord(sp.a, s);
}

hipError_t span_end(fluxmoe_ctx* c, hipStream_t s) {
    if (!c->span_open) return hipSuccess;
    c->span_open = false;
    return hipEventRecord(c->spans.back().b, s);
}

void ffn_span_hook(void* user, int kind, int begin, hipStream_t s) {
    fluxmoe_ctx* c = static_cast<fluxmoe_ctx*>(user);
    if (begin) (void)span_begin(c, kind, s); else (void)span_end(c, s);
}

}  // namespace

extern "C" {

const char* fluxmoe_last_error(void) { return g_err; }

int fluxmoe_create(const fluxmoe_desc* desc, fluxmoe_ctx** out_ctx) {
    if (!desc || !out_ctx) return set_error(FLUXMOE_EINVAL, "desc/out_ctx is NULL");
    fluxmoe_desc d = *desc;
    if (d.max_code_len == 0) d.max_code_len = 12;
    if (d.n_layers == 0 || d.n_experts == 0 || d.hidden == 0 || d.ffn == 0 || d.n_slots == 0)
        return set_error(FLUXMOE_EINVAL, "n_layers, n_experts, hidden, ffn, n_slots must be > 0");
    if (d.hidden % 8 || d.ffn % 8)
        return set_error(FLUXMOE_EINVAL, "hidden (%u) and ffn (%u) must be multiples of 8", d.hidden, d.ffn);
    if (d.block_bytes != 4096)
        return set_error(FLUXMOE_EINVAL, "block_bytes must be 4096 (got %u)", d.block_bytes);
    if (d.max_code_len < 8 || d.max_code_len > kLutBits)
        return set_error(FLUXMOE_EINVAL, "max_code_len must be in 8..12 (got %u)", d.max_code_len);
    if (d.flags != 0) return set_error(FLUXMOE_EINVAL, "flags must be 0");
    if (uint64_t(d.hidden) * d.ffn * 2 >= (1ull << 31))
        return set_error(FLUXMOE_EINVAL, "hidden * ffn * 2 bytes (one expert matrix) must stay under 2 GiB: "
                                         "the FFN kernels address a matrix with 32-bit byte offsets");
    if (d.n_experts > 4096) return set_error(FLUXMOE_EINVAL, "n_experts must be <= 4096");
    fluxmoe_ctx* c = new (std::nothrow) fluxmoe_ctx();
    if (!c) return set_error(FLUXMOE_ENOMEM, "out of host memory");
    c->d = d;
    c->elems2 = uint64_t(d.hidden) * d.ffn;
    c->elems13 = 2 * c->elems2;
    c->layers.resize(d.n_layers);
    c->pt.assign(size_t(d.n_layers) * d.n_experts, -1);
    c->slot_owner.assign(d.n_slots, -1);
    c->slot_last_reader.assign(d.n_slots, -1);
    c->load_valid.assign(d.n_layers, 0);
    c->infer_valid.assign(d.n_layers, 0);
    c->rel_valid.assign(d.n_layers, 0);
    compute_layout(c);
    if (const char* v = std::getenv("FLUXMOE_DECODE_WAVES")) {
        const int w = std::atoi(v);
        if (w == 4 || w == 8 || w == 16) c->tune_waves = w;
    }
    if (const char* v = std::getenv("FLUXMOE_DECODE_BLOCKS_PER_WAVE")) {
        const int w = std::atoi(v);
        if (w >= 1 && w <= 1024) c->tune_blocks_per_wave = w;
    }
    if (const char* v = std::getenv("FLUXMOE_FFN_TILED_WAVES")) {
        const int w = std::atoi(v);
        if (w == 1 || w == 2 || w == 4 || w == 8) c->tune_tiled_waves = w;
    }
    if (const char* v = std::getenv("FLUXMOE_FFN_TILED_PERSIST")) {
        const int w = std::atoi(v);
        if (w >= 0 && w <= 16) c->tune_tiled_persist = w;
    }
    if (const char* v = std::getenv("FLUXMOE_FFN_TILED_GROUP")) {
        const int w = std::atoi(v);
        if (w >= 1 && w <= 8) c->tune_tiled_group = w;
    }
    *out_ctx = c;
    g_err[0] = 0;
    return FLUXMOE_OK;
}

int fluxmoe_destroy(fluxmoe_ctx* c) {
    if (!c) return FLUXMOE_OK;
    if (c->events_ready) {
        for (auto e : c->ev_load) if (e) (void)hipEventDestroy(e);
        for (auto e : c->ev_infer) if (e) (void)hipEventDestroy(e);
        for (auto e : c->ev_rel) if (e) (void)hipEventDestroy(e);
        for (int i = 0; i < kRing; ++i) if (c->ring_ev[i]) (void)hipEventDestroy(c->ring_ev[i]);
        for (int i = 0; i < 2; ++i) if (c->ev_half_done[i]) (void)hipEventDestroy(c->ev_half_done[i]);
        for (int i = 0; i < 2; ++i) if (c->ev_copied[i]) (void)hipEventDestroy(c->ev_copied[i]);
        if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
        if (c->ev_join) (void)hipEventDestroy(c->ev_join);
        if (c->pinned_cmd) (void)hipHostFree(c->pinned_cmd);
    }
    delete c;
    return FLUXMOE_OK;
}

int fluxmoe_query_sizes(const fluxmoe_ctx* c, fluxmoe_sizes* out) {
    if (!c || !out) return set_error(FLUXMOE_EINVAL, "ctx/out is NULL");
    out->sigma1 = c->elems13 * 2;
    out->sigma2 = c->elems2 * 2;
    out->slots13_bytes = out->sigma1 * c->d.n_slots;
    out->slots2_bytes = out->sigma2 * c->d.n_slots;
    out->page_table_bytes = uint64_t(c->d.n_layers) * c->d.n_experts * 4;
    // worst case: every element costs 1 raw byte + max_code_len bits, plus headers and one
    // partly filled block per tensor
    const uint64_t per_block = c->d.block_bytes - kHeaderBytes;
    auto bound = [&](uint64_t elems) {
        const uint64_t bytes = elems + (elems * c->d.max_code_len + 7) / 8;
        return (bytes / (per_block - 8 * kGroup) + 2) * c->d.block_bytes;
    };
    out->layer_blob_bound = uint64_t(c->d.n_experts) * (bound(c->elems13) + bound(c->elems2));
    out->pool_workspace_bytes = c->pool_ws_bytes;
    return FLUXMOE_OK;
}

// extra scratch of the shared-expert call: its synthetic routing (ids, gates, one-entry table)
static uint64_t shared_extra_bytes(uint32_t T) { return 2 * align_up(uint64_t(T) * 4, 256) + 256; }

uint64_t fluxmoe_ffn_workspace_bytes(const fluxmoe_ctx* c, uint32_t T, uint32_t K, int shared_expert) {
    if (!c) return 0;
    uint64_t need = plan_ffn(ffn_shape(c, c->d.n_experts), T, K).bytes;
    if (shared_expert)          // same shapes, a single expert
        need = std::max(need, plan_ffn(ffn_shape(c, 1), T, 1).bytes + shared_extra_bytes(T));
    return need;
}

int fluxmoe_ffn_plan(const fluxmoe_ctx* c, uint32_t T, uint32_t K, uint32_t* rows_per_tile, uint32_t* k_splits) {
    if (!c || !rows_per_tile || !k_splits) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if (K == 0 || K > c->d.n_experts) return set_error(FLUXMOE_EINVAL, "K must be in 1..n_experts");
    const FfnPlan p = plan_ffn(ffn_shape(c, c->d.n_experts), T, K);
    *rows_per_tile = p.m_tile;
    *k_splits = p.ksplit;
    return FLUXMOE_OK;
}

int fluxmoe_encode_pool(fluxmoe_ctx* c, uint32_t layer, const uint16_t* w13, const uint16_t* w2,
                        void* dst, size_t dst_cap, size_t* dst_used, int n_threads) {
    if (int rc = check_layer(c, layer, false)) return rc;
    if (!w13 || !w2 || !dst || !dst_used) return set_error(FLUXMOE_EINVAL, "NULL argument");
    const uint32_t E = c->d.n_experts, B = c->d.block_bytes;
    n_threads = std::max(1, std::min(n_threads, 256));
    LayerMeta& L = c->layers[layer];
    L.encoded = false;
    L.bound = false;
    const uint64_t elems[2] = {c->elems13, c->elems2};
    const uint16_t* base[2] = {w13, w2};

    auto parallel_for = [&](uint32_t count, auto&& fn) {
        std::atomic<uint32_t> next{0};
        auto worker = [&]() {
            for (;;) {
                const uint32_t i = next.fetch_add(1);
                if (i >= count) break;
                fn(i);
            }
        };
        std::vector<std::thread> th;
        for (int t = 1; t < n_threads; ++t) th.emplace_back(worker);
        worker();
        for (auto& t : th) t.join();
    };

    // 1. exponent histograms, one per tensor type over all experts
    std::vector<std::array<uint64_t, 256>> hist(2 * size_t(E));
    parallel_for(2 * E, [&](uint32_t i) {
        const int ti = i / E;
        const uint32_t e = i % E;
        auto& h = hist[i];
        h.fill(0);
        const uint16_t* w = base[ti] + size_t(e) * elems[ti];
        uint64_t local[4][256] = {};
        uint64_t m = 0;
        for (; m + 4 <= elems[ti]; m += 4) {
            ++local[0][(w[m] >> 7) & 0xFF];
            ++local[1][(w[m + 1] >> 7) & 0xFF];
            ++local[2][(w[m + 2] >> 7) & 0xFF];
            ++local[3][(w[m + 3] >> 7) & 0xFF];
        }
        for (; m < elems[ti]; ++m) ++local[0][(w[m] >> 7) & 0xFF];
        for (int s = 0; s < 256; ++s) h[s] = local[0][s] + local[1][s] + local[2][s] + local[3][s];
    });
    uint16_t codes[2][256];
    for (int ti = 0; ti < 2; ++ti) {
        uint64_t total[256] = {};
        for (uint32_t e = 0; e < E; ++e)
            for (int s = 0; s < 256; ++s) total[s] += hist[size_t(ti) * E + e][s];
        limited_code_lengths(total, c->d.max_code_len, L.lens[ti]);
        canonical_codes(L.lens[ti], codes[ti]);
        L.payload_bits[ti] = 0;
        for (int s = 0; s < 256; ++s) L.payload_bits[ti] += total[s] * L.lens[ti][s];
        L.tensors[ti].assign(E, TensorMeta());
    }
    // 2. block plan of every tensor
    parallel_for(2 * E, [&](uint32_t i) {
        const int ti = i / E;
        const uint32_t e = i % E;
        plan_tensor(base[ti] + size_t(e) * elems[ti], elems[ti], L.lens[ti], B,
                    L.tensors[ti][e].first_elem);
    });
    // 3. blob order: down tensors (type 2) first, then fused gate/up tensors
    uint64_t nb = 0;
    for (int ti : {1, 0})
        for (uint32_t e = 0; e < E; ++e) {
            L.tensors[ti][e].first_block = nb;
            nb += L.tensors[ti][e].n_blocks();
        }
    L.n_blocks = nb;
    *dst_used = size_t(nb) * B;
    if (size_t(nb) * B > dst_cap)
        return set_error(FLUXMOE_ENOMEM, "layer blob needs %zu bytes, dst_cap is %zu", size_t(nb) * B, dst_cap);
    // 4. encode
    uint8_t* out = static_cast<uint8_t*>(dst);
    parallel_for(2 * E, [&](uint32_t i) {
        const int ti = i / E;
        const uint32_t e = i % E;
        const TensorMeta& tm = L.tensors[ti][e];
        encode_tensor(base[ti] + size_t(e) * elems[ti], tm.first_elem, L.lens[ti], codes[ti], B,
                      out + size_t(tm.first_block) * B);
    });
    L.encoded = true;
    return FLUXMOE_OK;
}

int fluxmoe_layer_info_get(const fluxmoe_ctx* c, uint32_t layer, fluxmoe_layer_info* out) {
    if (int rc = check_layer(c, layer, true)) return rc;
    if (!out) return set_error(FLUXMOE_EINVAL, "out is NULL");
    const LayerMeta& L = c->layers[layer];
    out->n_blocks = L.n_blocks;
    out->payload_bits[0] = L.payload_bits[0];
    out->payload_bits[1] = L.payload_bits[1];
    out->elements[0] = c->elems13 * c->d.n_experts;
    out->elements[1] = c->elems2 * c->d.n_experts;
    return FLUXMOE_OK;
}

static int type_index(int type) { return type == 1 ? 0 : (type == 2 ? 1 : -1); }

int fluxmoe_code_lengths(const fluxmoe_ctx* c, uint32_t layer, int type, uint8_t out_lens[256]) {
    if (int rc = check_layer(c, layer, true)) return rc;
    const int ti = type_index(type);
    if (ti < 0 || !out_lens) return set_error(FLUXMOE_EINVAL, "type must be 1 or 2, out non-NULL");
    std::memcpy(out_lens, c->layers[layer].lens[ti], 256);
    return FLUXMOE_OK;
}

int fluxmoe_tensor_blocks(const fluxmoe_ctx* c, uint32_t layer, int type, uint32_t expert,
                          uint64_t* first_block, uint64_t* n_blocks) {
    if (int rc = check_layer(c, layer, true)) return rc;
    const int ti = type_index(type);
    if (ti < 0 || !first_block || !n_blocks) return set_error(FLUXMOE_EINVAL, "bad type or NULL out");
    if (expert >= c->d.n_experts) return set_error(FLUXMOE_ERANGE, "expert %u out of range", expert);
    const TensorMeta& tm = c->layers[layer].tensors[ti][expert];
    *first_block = tm.first_block;
    *n_blocks = tm.n_blocks();
    return FLUXMOE_OK;
}

int fluxmoe_tensor_first_elems(const fluxmoe_ctx* c, uint32_t layer, int type, uint32_t expert,
                               uint32_t* out, size_t out_cap) {
    if (int rc = check_layer(c, layer, true)) return rc;
    const int ti = type_index(type);
    if (ti < 0 || !out) return set_error(FLUXMOE_EINVAL, "bad type or NULL out");
    if (expert >= c->d.n_experts) return set_error(FLUXMOE_ERANGE, "expert %u out of range", expert);
    const TensorMeta& tm = c->layers[layer].tensors[ti][expert];
    if (out_cap < tm.first_elem.size())
        return set_error(FLUXMOE_ENOMEM, "out_cap %zu < %zu", out_cap, tm.first_elem.size());
    std::memcpy(out, tm.first_elem.data(), tm.first_elem.size() * 4);
    return FLUXMOE_OK;
}

int fluxmoe_bind_arenas(fluxmoe_ctx* c, void* slots13, void* slots2, void* workspace,
                        size_t workspace_bytes) {
    if (!c) return set_error(FLUXMOE_EINVAL, "ctx is NULL");
    if (!slots13 || !slots2 || !workspace) return set_error(FLUXMOE_EINVAL, "NULL arena");
    if ((uintptr_t(slots13) | uintptr_t(slots2) | uintptr_t(workspace)) & 255)
        return set_error(FLUXMOE_EINVAL, "arenas must be 256-byte aligned");
    if (workspace_bytes < c->pool_ws_bytes)
        return set_error(FLUXMOE_ENOMEM, "workspace needs at least %llu bytes",
                         (unsigned long long)c->pool_ws_bytes);
    int dev = 0;
    HIPCHECK(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIPCHECK(hipGetDeviceProperties(&prop, dev));
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return set_error(FLUXMOE_EHIP, "device is %s; this library is built for gfx950 only", prop.gcnArchName);
    c->n_cus = prop.multiProcessorCount;
    if (int rc = resolve_static_scratch(dev)) return rc;
    c->device = dev;
    if (int rc = ensure_events(c)) return rc;
    c->slots13 = static_cast<uint8_t*>(slots13);
    c->slots2 = static_cast<uint8_t*>(slots2);
    c->ws = static_cast<uint8_t*>(workspace);
    c->ws_bytes = workspace_bytes;
    HIPCHECK(hipMemset(c->ws + c->err_off, 0, 256));
    c->arenas_bound = true;
    for (auto& L : c->layers) L.bound = false;
    return FLUXMOE_OK;
}

int fluxmoe_bind_layer(fluxmoe_ctx* c, uint32_t layer, const void* hbm_blocks, uint64_t n_host_blocks,
                       const void* host_blocks, const void* check_host_copy) {
    if (int rc = check_layer(c, layer, true)) return rc;
    if (!c->arenas_bound) return set_error(FLUXMOE_ESTATE, "fluxmoe_bind_arenas has not been called");
    LayerMeta& L = c->layers[layer];
    if (n_host_blocks > L.n_blocks)
        return set_error(FLUXMOE_ERANGE, "n_host_blocks %llu > n_blocks %llu",
                         (unsigned long long)n_host_blocks, (unsigned long long)L.n_blocks);
    if (n_host_blocks > 0 && !host_blocks) return set_error(FLUXMOE_EINVAL, "host_blocks is NULL");
    if (n_host_blocks < L.n_blocks && !hbm_blocks) return set_error(FLUXMOE_EINVAL, "hbm_blocks is NULL");
    if ((uintptr_t(hbm_blocks) | uintptr_t(host_blocks)) & 15)
        return set_error(FLUXMOE_EINVAL, "block arenas must be 16-byte aligned");
    if (check_host_copy) {
        const uint8_t* blob = static_cast<const uint8_t*>(check_host_copy);
        const uint32_t B = c->d.block_bytes;
        for (int ti = 0; ti < 2; ++ti)
            for (uint32_t e = 0; e < c->d.n_experts; ++e) {
                const TensorMeta& tm = L.tensors[ti][e];
                for (uint64_t k = 0; k < tm.n_blocks(); ++k) {
                    uint32_t hdr[2];
                    std::memcpy(hdr, blob + (tm.first_block + k) * B, 8);
                    if (hdr[0] != tm.first_elem[k + 1] - tm.first_elem[k] || hdr[1] != tm.first_elem[k])
                        return set_error(FLUXMOE_ECORRUPT,
                                         "layer %u type %d expert %u block %llu: header (n=%u, e0=%u) "
                                         "does not match the encoder's metadata",
                                         layer, ti + 1, e, (unsigned long long)k, hdr[0], hdr[1]);
                }
            }
    }
    std::vector<uint32_t> lut(2 * kLutEntries);
    build_lut(L.lens[0], lut.data());
    build_lut(L.lens[1], lut.data() + kLutEntries);
    HIPCHECK(hipMemcpy(c->ws + c->lut_off + uint64_t(layer) * 2 * kLutBytes, lut.data(), 2 * kLutBytes,
                       hipMemcpyHostToDevice));
    L.hbm = static_cast<const uint8_t*>(hbm_blocks);
    L.host = static_cast<const uint8_t*>(host_blocks);
    L.n_host_blocks = n_host_blocks;
    L.host_tensors = 0;
    for (int ti = 0; ti < 2; ++ti)
        for (TensorMeta& tm : L.tensors[ti]) {
            const uint64_t a = tm.first_block, b = a + tm.n_blocks();
            const uint64_t hb = std::min(b, std::max(a, n_host_blocks));
            tm.n_host = hb - a;
            tm.raw_src = nullptr;
            tm.host_src = tm.n_host ? L.host + a * c->d.block_bytes : nullptr;
            tm.hbm_src = hb < b ? L.hbm + (hb - n_host_blocks) * c->d.block_bytes : nullptr;
            L.host_tensors += tm.on_host() ? 1 : 0;
        }
    L.bound = true;
    if (c->half[layer & 1].layer == int64_t(layer)) c->half[layer & 1].layer = -1;
    return FLUXMOE_OK;
}

int fluxmoe_bind_staging(fluxmoe_ctx* c, void* staging, size_t staging_bytes) {
    if (!c) return set_error(FLUXMOE_EINVAL, "ctx is NULL");
    if (!staging || (uintptr_t(staging) & 255)) return set_error(FLUXMOE_EINVAL, "staging must be non-NULL, 256-byte aligned");
    if (staging_bytes < 2ull * c->d.block_bytes) return set_error(FLUXMOE_ENOMEM, "staging too small");
    c->staging = static_cast<uint8_t*>(staging);
    c->staging_bytes = staging_bytes;
    c->half[0].layer = c->half[1].layer = -1;
    return FLUXMOE_OK;
}

int fluxmoe_set_tensor_backing(fluxmoe_ctx* c, uint32_t layer, int type, uint32_t expert, int tier,
                               const void* blocks) {
    if (int rc = check_layer(c, layer, true)) return rc;
    LayerMeta& L = c->layers[layer];
    if (!L.bound) return set_error(FLUXMOE_ESTATE, "layer %u is not bound", layer);
    if (type != 1 && type != 2) return set_error(FLUXMOE_EINVAL, "type must be 1 or 2");
    if (expert >= c->d.n_experts) return set_error(FLUXMOE_ERANGE, "expert %u out of range", expert);
    if (tier != FLUXMOE_TIER_HBM && tier != FLUXMOE_TIER_HOST && tier != FLUXMOE_TIER_HOST_RAW)
        return set_error(FLUXMOE_EINVAL, "tier must be 0 (HBM), 1 (pinned host, compressed) or 2 (pinned host, dense)");
    if (!blocks || (uintptr_t(blocks) & 15)) return set_error(FLUXMOE_EINVAL, "blocks must be non-NULL, 16-byte aligned");
    TensorMeta& tm = L.tensors[type - 1][expert];
    L.host_tensors -= tm.on_host() ? 1 : 0;
    tm.n_host = 0;
    tm.host_src = tm.hbm_src = tm.raw_src = nullptr;
    if (tier == FLUXMOE_TIER_HOST) {
        tm.n_host = tm.n_blocks();
        tm.host_src = static_cast<const uint8_t*>(blocks);
    } else if (tier == FLUXMOE_TIER_HOST_RAW) {
        tm.raw_src = static_cast<const uint8_t*>(blocks);
    } else {
        tm.hbm_src = static_cast<const uint8_t*>(blocks);
    }
    L.host_tensors += tm.on_host() ? 1 : 0;
    if (c->half[layer & 1].layer == int64_t(layer)) c->half[layer & 1].layer = -1;   // staged copies are stale
    return FLUXMOE_OK;
}

int fluxmoe_reset_page_table(fluxmoe_ctx* c, int32_t* page_table, void* stream) {
    if (!c || !page_table) return set_error(FLUXMOE_EINVAL, "NULL argument");
    HIPCHECK(launch_fill_i32(page_table, -1, uint64_t(c->d.n_layers) * c->d.n_experts,
                             static_cast<hipStream_t>(stream)));
    std::fill(c->pt.begin(), c->pt.end(), -1);
    std::fill(c->slot_owner.begin(), c->slot_owner.end(), -1);
    return FLUXMOE_OK;
}

static int validate_ids(const fluxmoe_ctx* c, const int32_t* ids, uint32_t n) {
    if (n > c->d.n_experts) return set_error(FLUXMOE_EINVAL, "n %u > n_experts %u", n, c->d.n_experts);
    if (n && !ids) return set_error(FLUXMOE_EINVAL, "expert_ids is NULL");
    std::vector<uint8_t> seen(c->d.n_experts, 0);
    for (uint32_t i = 0; i < n; ++i) {
        if (ids[i] < 0 || uint32_t(ids[i]) >= c->d.n_experts)
            return set_error(FLUXMOE_ERANGE, "expert id %d out of range [0, %u)", ids[i], c->d.n_experts);
        if (seen[ids[i]]++) return set_error(FLUXMOE_EINVAL, "expert id %d listed twice", ids[i]);
    }
    return FLUXMOE_OK;
}

// Copies of the listed experts' host-tier blocks into the layer's staging half (layer & 1).
// The half keeps them until the next staging into it; the copies wait (on the device) for the
// last decode that read the half.
static int stage_host_blocks(fluxmoe_ctx* c, uint32_t layer, const int32_t* ids, uint32_t n,
                             hipStream_t s) {
    LayerMeta& L = c->layers[layer];
    const int h = layer & 1;
    StageHalf& st = c->half[h];
    st.layer = -1;
    st.off[0].assign(c->d.n_experts, -1);
    st.off[1].assign(c->d.n_experts, -1);
    if (L.host_tensors == 0) { st.layer = layer; return FLUXMOE_OK; }
    if (!c->staging) return set_error(FLUXMOE_ESTATE, "layer %u has host-tier blocks but no staging buffer is bound", layer);
    const uint32_t B = c->d.block_bytes;
    const uint64_t half_bytes = (c->staging_bytes / 2) / B * B;
    uint8_t* base = c->staging + h * half_bytes;
    std::vector<int32_t> sorted(ids, ids + n);
    std::sort(sorted.begin(), sorted.end());
    struct Range { const uint8_t* src; uint64_t bytes, dst; };
    std::vector<Range> ranges;               // adjacent source ranges are merged into one copy
    uint64_t cursor = 0;
    for (int ti : {1, 0})
        for (int32_t e : sorted) {
            const TensorMeta& tm = L.tensors[ti][e];
            if (!tm.on_host()) continue;
            st.off[ti][e] = int64_t(cursor);
            // dense tensors are staged whole (a multiple of 16 bytes); the cursor stays block aligned
            const uint8_t* src = tm.raw_src ? tm.raw_src : tm.host_src;
            const uint64_t bytes = tm.raw_src ? (ti == 0 ? c->elems13 : c->elems2) * 2 : tm.n_host * B;
            if (!ranges.empty() && ranges.back().src + ranges.back().bytes == src &&
                ranges.back().dst + ranges.back().bytes == cursor) ranges.back().bytes += bytes;
            else ranges.push_back({src, bytes, cursor});
            cursor += align_up(bytes, B);
        }
    if (cursor > half_bytes)
        return set_error(FLUXMOE_ENOMEM, "staging half holds %llu bytes, layer %u needs %llu",
                         (unsigned long long)half_bytes, layer, (unsigned long long)cursor);
    if (c->half_done_valid[h]) HIPCHECK(hipStreamWaitEvent(s, c->ev_half_done[h], 0));
    // an earlier staging into this half may have been issued on another stream (a prefetch on the copy
    // stream, then a materialize of other experts that restages on its own stream): its copies must
    // have landed before these overwrite the half with a different layout
    if (c->copied_valid[h]) HIPCHECK(hipStreamWaitEvent(s, c->ev_copied[h], 0));
    for (const Range& r : ranges)
        HIPCHECK(hipMemcpyAsync(base + r.dst, r.src, r.bytes, hipMemcpyHostToDevice, s));
    HIPCHECK(hipEventRecord(c->ev_copied[h], s));
    c->copied_valid[h] = true;
    st.layer = layer;
    return FLUXMOE_OK;
}

int fluxmoe_prefetch_host(fluxmoe_ctx* c, uint32_t layer, const int32_t* expert_ids, uint32_t n,
                          void* copy_stream) {
    if (int rc = check_layer(c, layer, true)) return rc;
    if (!c->layers[layer].bound) return set_error(FLUXMOE_ESTATE, "layer %u is not bound", layer);
    if (int rc = validate_ids(c, expert_ids, n)) return rc;
    return stage_host_blocks(c, layer, expert_ids, n, static_cast<hipStream_t>(copy_stream));
}

// Body of fluxmoe_materialize and fluxmoe_materialize_two_streams.  two_streams: the down tensors (type 2) are
// decoded on stream2_v while the fused gate/up tensors (type 1) are decoded on stream_v; stream_v waits for
// both before it records the layer's load event.
static int materialize_enqueue(fluxmoe_ctx* c, uint32_t layer, const int32_t* expert_ids, uint32_t n,
                               int32_t* page_table, const int32_t* dst_slots, void* stream_v, bool two_streams,
                               void* stream2_v) {
    if (int rc = check_layer(c, layer, true)) return rc;
    LayerMeta& L = c->layers[layer];
    if (!c->arenas_bound || !L.bound) return set_error(FLUXMOE_ESTATE, "arenas or layer %u not bound", layer);
    if (!page_table) return set_error(FLUXMOE_EINVAL, "page_table is NULL");
    if (int rc = validate_ids(c, expert_ids, n)) return rc;
    if (n && !dst_slots) return set_error(FLUXMOE_EINVAL, "dst_slots is NULL");
    {
        std::vector<uint8_t> seen(c->d.n_slots, 0);
        for (uint32_t i = 0; i < n; ++i) {
            if (dst_slots[i] < 0 || uint32_t(dst_slots[i]) >= c->d.n_slots)
                return set_error(FLUXMOE_ERANGE, "slot %d out of range [0, %u)", dst_slots[i], c->d.n_slots);
            if (seen[dst_slots[i]]++) return set_error(FLUXMOE_EINVAL, "slot %d listed twice", dst_slots[i]);
        }
    }
    if (n == 0) return FLUXMOE_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const uint32_t E = c->d.n_experts, B = c->d.block_bytes;

    // host-tier parts must be staged for exactly these experts
    bool need_host = false;
    for (uint32_t i = 0; i < n && !need_host; ++i)
        for (int ti = 0; ti < 2; ++ti)
            if (L.tensors[ti][expert_ids[i]].on_host()) need_host = true;
    bool wait_copy = false;
    if (need_host) {
        StageHalf& st = c->half[layer & 1];
        bool staged = st.layer == int64_t(layer);
        for (uint32_t i = 0; i < n && staged; ++i)
            for (int ti = 0; ti < 2; ++ti)
                if (L.tensors[ti][expert_ids[i]].on_host() && st.off[ti][expert_ids[i]] < 0)
                    staged = false;
        if (!staged) {
            if (int rc = stage_host_blocks(c, layer, expert_ids, n, stream)) return rc;
        } else {
            wait_copy = true;
        }
    }

    // ring slot for the command buffer
    const int slot = c->ring_next;
    if (c->ring_used[slot]) HIPCHECK(hipEventSynchronize(c->ring_ev[slot]));
    uint8_t* hcmd = c->pinned_cmd + size_t(slot) * c->cmd_bytes;
    uint8_t* dcmd = c->ws + c->cmd_off + size_t(slot) * c->cmd_bytes;
    DecodeCmd* cmd = reinterpret_cast<DecodeCmd*>(hcmd);
    const uint32_t jobs_off[2] = {uint32_t(sizeof(DecodeCmd)),
                                  uint32_t(sizeof(DecodeCmd) + c->max_jobs * sizeof(DecodeJob))};
    const uint32_t upd_off = uint32_t(sizeof(DecodeCmd) + 2ull * c->max_jobs * sizeof(DecodeJob));
    std::memset(cmd, 0, sizeof(DecodeCmd));

    const int half = layer & 1;
    const uint64_t half_bytes = c->staging ? (c->staging_bytes / 2) / B * B : 0;
    struct DenseCopy { const uint8_t* src; uint8_t* dst; uint64_t bytes; };
    std::vector<DenseCopy> dense_copies;     // staged uncompressed tensors: staging -> slot, no decode
    for (int ti = 0; ti < 2; ++ti) {
        DecodeJob* jobs = reinterpret_cast<DecodeJob*>(hcmd + jobs_off[ti]);
        uint32_t nj = 0, blocks = 0;
        const uint64_t sigma = (ti == 0 ? c->elems13 : c->elems2) * 2;
        uint8_t* arena = ti == 0 ? c->slots13 : c->slots2;
        for (uint32_t i = 0; i < n; ++i) {
            const TensorMeta& tm = L.tensors[ti][expert_ids[i]];
            const uint64_t nb = tm.n_blocks(), nh = tm.n_host;     // host part is the first nh blocks
            const uint64_t dst = uint64_t(uintptr_t(arena)) + uint64_t(dst_slots[i]) * sigma;
            if (tm.raw_src) {
                dense_copies.push_back({c->staging + half * half_bytes + c->half[half].off[ti][expert_ids[i]],
                                        reinterpret_cast<uint8_t*>(uintptr_t(dst)), sigma});
                continue;
            }
            if (nh) {
                const uint8_t* src = c->staging + half * half_bytes + c->half[half].off[ti][expert_ids[i]];
                jobs[nj++] = DecodeJob{uint64_t(uintptr_t(src)), dst, blocks, uint32_t(nh),
                                       uint32_t(ti == 0 ? c->elems13 : c->elems2), 0};
                blocks += uint32_t(nh);
            }
            if (nb > nh) {
                jobs[nj++] = DecodeJob{uint64_t(uintptr_t(tm.hbm_src)), dst, blocks, uint32_t(nb - nh),
                                       uint32_t(ti == 0 ? c->elems13 : c->elems2), 0};
                blocks += uint32_t(nb - nh);
            }
        }
        cmd->n_jobs[ti] = nj;
        cmd->total_blocks[ti] = blocks;
    }

    // page-table transitions on the host mirror; the touched entries go to the device
    std::vector<int64_t> touched;
    std::vector<int32_t> wait_layers;
    for (uint32_t i = 0; i < n; ++i) {
        const int64_t key = int64_t(layer) * E + expert_ids[i];
        const int32_t s = dst_slots[i];
        const int32_t old_slot = c->pt[key];
        if (old_slot >= 0 && old_slot != s) c->slot_owner[old_slot] = -1;
        const int64_t prev = c->slot_owner[s];
        if (prev >= 0 && prev != key) {
            c->pt[prev] = -1;
            touched.push_back(prev);
        }
        c->pt[key] = s;
        c->slot_owner[s] = key;
        touched.push_back(key);
        const int32_t lr = c->slot_last_reader[s];
        if (lr >= 0 && c->infer_valid[lr] &&
            std::find(wait_layers.begin(), wait_layers.end(), lr) == wait_layers.end())
            wait_layers.push_back(lr);
        c->slot_last_reader[s] = -1;
    }
    std::sort(touched.begin(), touched.end());
    touched.erase(std::unique(touched.begin(), touched.end()), touched.end());
    int32_t* upd = reinterpret_cast<int32_t*>(hcmd + upd_off);
    for (size_t i = 0; i < touched.size(); ++i) {
        upd[2 * i] = int32_t(touched[i]);
        upd[2 * i + 1] = c->pt[touched[i]];
    }
    cmd->n_pt_updates = uint32_t(touched.size());

    // enqueue: WAR waits, host-tier copies, command upload, decode, events
    for (int32_t lr : wait_layers) HIPCHECK(hipStreamWaitEvent(stream, c->ev_infer[lr], 0));
    // a release of this layer issued on another stream writes the same page-table row
    if (c->rel_valid[layer]) HIPCHECK(hipStreamWaitEvent(stream, c->ev_rel[layer], 0));
    if (wait_copy) HIPCHECK(hipStreamWaitEvent(stream, c->ev_copied[half], 0));

    DecodeArgs args{};
    args.lut[0] = reinterpret_cast<const uint32_t*>(c->ws + c->lut_off + (uint64_t(layer) * 2 + 0) * kLutBytes);
    args.lut[1] = reinterpret_cast<const uint32_t*>(c->ws + c->lut_off + (uint64_t(layer) * 2 + 1) * kLutBytes);
    args.page_table = page_table;
    args.error_word = reinterpret_cast<uint32_t*>(c->ws + c->err_off);
    // A command that is small enough travels inside the kernel arguments, packed without the gaps of the
    // ring slot's fixed layout; a larger one is uploaded into the ring slot in front of the kernel.
    const uint64_t decode_blocks = uint64_t(cmd->total_blocks[0]) + cmd->total_blocks[1];
    const size_t jobs_bytes[2] = {cmd->n_jobs[0] * sizeof(DecodeJob), cmd->n_jobs[1] * sizeof(DecodeJob)};
    const size_t packed = sizeof(DecodeCmd) + jobs_bytes[0] + jobs_bytes[1] + touched.size() * 8;
    if (decode_blocks > 0 && packed <= kInlineCmdBytes) {
        uint8_t* w = reinterpret_cast<uint8_t*>(args.inline_words);
        std::memcpy(w, cmd, sizeof(DecodeCmd));
        args.jobs_offset[0] = uint32_t(sizeof(DecodeCmd));
        args.jobs_offset[1] = uint32_t(args.jobs_offset[0] + jobs_bytes[0]);
        args.upd_offset = uint32_t(args.jobs_offset[1] + jobs_bytes[1]);
        std::memcpy(w + args.jobs_offset[0], hcmd + jobs_off[0], jobs_bytes[0]);
        std::memcpy(w + args.jobs_offset[1], hcmd + jobs_off[1], jobs_bytes[1]);
        std::memcpy(w + args.upd_offset, hcmd + upd_off, touched.size() * 8);
        args.inline_cmd = 1;
        args.cmd = nullptr;
    } else {
        const size_t used = upd_off + touched.size() * 8;
        HIPCHECK(hipMemcpyAsync(dcmd, hcmd, used, hipMemcpyHostToDevice, stream));
        args.cmd = reinterpret_cast<const DecodeCmd*>(dcmd);
        args.jobs_offset[0] = jobs_off[0];
        args.jobs_offset[1] = jobs_off[1];
        args.upd_offset = upd_off;
        args.inline_cmd = 0;
    }
    for (const DenseCopy& dc : dense_copies)
        HIPCHECK(hipMemcpyAsync(dc.dst, dc.src, dc.bytes, hipMemcpyDeviceToDevice, stream));
    const int waves_per_wg = c->tune_waves;
    const uint64_t total = uint64_t(cmd->total_blocks[0]) + cmd->total_blocks[1];
    if (total == 0) {
        // every listed tensor is an uncompressed host tensor: nothing to decode, only the page table changes
        if (!touched.empty())
            HIPCHECK(launch_apply_updates(page_table, dcmd + upd_off, uint32_t(touched.size()), stream));
    } else {
    // blocks per workgroup: a few per wavefront, fewer when that would leave CUs without work
    const uint64_t fill = total / (3ull * uint64_t(std::max(c->n_cus, 1)));
    const uint64_t per_wg = std::max<uint64_t>(waves_per_wg, std::min<uint64_t>(uint64_t(waves_per_wg) * c->tune_blocks_per_wave, fill));
    auto wgs_for = [&](uint64_t blocks) { return uint32_t(std::min<uint64_t>((blocks + per_wg - 1) / per_wg, 1u << 20)); };
    if (two_streams && cmd->total_blocks[0] && cmd->total_blocks[1]) {
        // one launch per tensor type: the type-2 list on the second stream (after everything this call has
        // enqueued on the first one so far), the type-1 list and the page-table updates on the first
        hipStream_t stream2 = static_cast<hipStream_t>(stream2_v);
        HIPCHECK(hipEventRecord(c->ev_fork, stream));
        HIPCHECK(hipStreamWaitEvent(stream2, c->ev_fork, 0));
        DecodeArgs a2 = args;
        const uint32_t n2 = wgs_for(cmd->total_blocks[1]);
        a2.wg_split = n2;                       // every workgroup serves the type-2 list
        a2.apply_updates = 0;
        HIPCHECK(launch_decode(a2, n2, waves_per_wg, stream2));
        HIPCHECK(hipEventRecord(c->ev_join, stream2));
        args.wg_split = 0;                      // every workgroup serves the type-1 list
        args.apply_updates = 1;
        HIPCHECK(span_begin(c, 0, stream));
        HIPCHECK(launch_decode(args, wgs_for(cmd->total_blocks[0]), waves_per_wg, stream));
        HIPCHECK(span_end(c, stream));
        HIPCHECK(hipStreamWaitEvent(stream, c->ev_join, 0));
    } else {
        uint32_t n_wg = std::max(wgs_for(total), 2u);
        uint32_t split = uint32_t((uint64_t(n_wg) * cmd->total_blocks[1] + total / 2) / total);
        split = std::min(std::max(split, 1u), n_wg - 1);
        args.wg_split = split;
        args.apply_updates = 1;
        HIPCHECK(span_begin(c, 0, stream));
        HIPCHECK(launch_decode(args, n_wg, waves_per_wg, stream));
        HIPCHECK(span_end(c, stream));
    }
    }
    HIPCHECK(hipEventRecord(c->ring_ev[slot], stream));
    c->ring_used[slot] = true;
    c->ring_next = (slot + 1) % kRing;
    if (need_host) {
        HIPCHECK(hipEventRecord(c->ev_half_done[half], stream));
        c->half_done_valid[half] = true;
    }
    HIPCHECK(hipEventRecord(c->ev_load[layer], stream));
    c->load_valid[layer] = 1;
    return FLUXMOE_OK;
}

int fluxmoe_materialize(fluxmoe_ctx* c, uint32_t layer, const int32_t* expert_ids, uint32_t n,
                        int32_t* page_table, const int32_t* dst_slots, void* stream) {
    return materialize_enqueue(c, layer, expert_ids, n, page_table, dst_slots, stream, false, nullptr);
}

int fluxmoe_materialize_two_streams(fluxmoe_ctx* c, uint32_t layer, const int32_t* expert_ids, uint32_t n,
                                    int32_t* page_table, const int32_t* dst_slots, void* stream,
                                    void* stream_type2) {
    return materialize_enqueue(c, layer, expert_ids, n, page_table, dst_slots, stream, stream_type2 != stream, stream_type2);
}

int fluxmoe_release(fluxmoe_ctx* c, uint32_t layer, const int32_t* expert_ids, uint32_t n,
                    int32_t* page_table, void* stream_v) {
    if (int rc = check_layer(c, layer, false)) return rc;
    if (!c->arenas_bound) return set_error(FLUXMOE_ESTATE, "fluxmoe_bind_arenas has not been called");
    if (!page_table) return set_error(FLUXMOE_EINVAL, "page_table is NULL");
    if (expert_ids) {
        if (int rc = validate_ids(c, expert_ids, n)) return rc;
    } else if (n != 0) {
        return set_error(FLUXMOE_EINVAL, "expert_ids is NULL but n is %u", n);
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const uint32_t E = c->d.n_experts;
    const int slot = c->ring_next;
    if (c->ring_used[slot]) HIPCHECK(hipEventSynchronize(c->ring_ev[slot]));
    uint8_t* hcmd = c->pinned_cmd + size_t(slot) * c->cmd_bytes;
    uint8_t* dcmd = c->ws + c->cmd_off + size_t(slot) * c->cmd_bytes;
    int32_t* upd = reinterpret_cast<int32_t*>(hcmd);
    uint32_t m = 0;
    const uint32_t count = expert_ids ? n : E;
    for (uint32_t i = 0; i < count; ++i) {
        const int64_t key = int64_t(layer) * E + (expert_ids ? expert_ids[i] : int32_t(i));
        const int32_t s = c->pt[key];
        if (s < 0) continue;
        c->pt[key] = -1;
        c->slot_owner[s] = -1;       // the slot keeps its last-reader layer: reuse still waits
        upd[2 * m] = int32_t(key);
        upd[2 * m + 1] = -1;
        ++m;
    }
    if (m == 0) return FLUXMOE_OK;
    // the entries are read by the layer's FFN and written by its materialize, possibly on other streams
    if (c->infer_valid[layer]) HIPCHECK(hipStreamWaitEvent(stream, c->ev_infer[layer], 0));
    if (c->load_valid[layer]) HIPCHECK(hipStreamWaitEvent(stream, c->ev_load[layer], 0));
    if (m <= kInlineUpdates) {
        HIPCHECK(launch_apply_updates_inline(page_table, upd, m, stream));     // the pairs travel in the kernel arguments
    } else {
        HIPCHECK(hipMemcpyAsync(dcmd, hcmd, size_t(m) * 8, hipMemcpyHostToDevice, stream));
        HIPCHECK(launch_apply_updates(page_table, dcmd, m, stream));
    }
    HIPCHECK(hipEventRecord(c->ev_rel[layer], stream));
    c->rel_valid[layer] = 1;
    HIPCHECK(hipEventRecord(c->ring_ev[slot], stream));
    c->ring_used[slot] = true;
    c->ring_next = (slot + 1) % kRing;
    return FLUXMOE_OK;
}

// Shared body of fluxmoe_expert_ffn and fluxmoe_expert_ffn_static: `w` is the FFN scratch (pair order, tile
// list, h, split-K partials) of `w_bytes` bytes, `w_name` says where it comes from in error texts.
static int expert_ffn_enqueue(fluxmoe_ctx* c, uint32_t layer, const uint16_t* tokens, uint32_t T,
                              const int32_t* topk_ids, const float* topk_w, uint32_t K,
                              const int32_t* page_table, float* out, uint32_t flags, void* stream_v,
                              uint8_t* w, uint64_t w_bytes, const char* w_name) {
    if (!tokens || !topk_ids || !topk_w || !page_table || !out) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if (K == 0 || K > c->d.n_experts) return set_error(FLUXMOE_EINVAL, "K must be in 1..n_experts");
    if (flags & ~3u) return set_error(FLUXMOE_EINVAL, "unknown flags 0x%x", flags);
    if (uint64_t(T) * K >= (1ull << 31) || T > 65535) return set_error(FLUXMOE_EINVAL, "T too large");
    if (uint64_t(T) * c->d.hidden * 2 >= (1ull << 32))
        return set_error(FLUXMOE_EINVAL, "tokens (T * hidden * 2 bytes) must stay under 4 GiB");
    if ((uintptr_t(tokens) | uintptr_t(out)) & 15) return set_error(FLUXMOE_EINVAL, "tokens/out must be 16-byte aligned");
    const FfnPlan p = plan_ffn(ffn_shape(c, c->d.n_experts), T, K);
    if (p.bytes > w_bytes)
        return set_error(FLUXMOE_ENOMEM, "%s holds %llu bytes, T=%u K=%u needs %llu", w_name,
                         (unsigned long long)w_bytes, T, K, (unsigned long long)p.bytes);
    if (p.tiles_cap > 65535) return set_error(FLUXMOE_EINVAL, "too many row tiles (%u)", p.tiles_cap);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    FfnArgs a{};
    a.tokens = tokens;
    a.topk_ids = topk_ids;
    a.topk_w = topk_w;
    a.page_table = page_table + size_t(layer) * c->d.n_experts;
    a.slots13 = reinterpret_cast<const uint16_t*>(c->slots13);
    a.slots2 = reinterpret_cast<const uint16_t*>(c->slots2);
    a.out = out;
    a.T = T; a.K = K; a.H = c->d.hidden; a.F = c->d.ffn; a.E = c->d.n_experts;
    a.flags = flags;
    a.expert_count = reinterpret_cast<int32_t*>(w + p.off_count);
    a.expert_offset = reinterpret_cast<int32_t*>(w + p.off_offset);
    a.sorted_pair = reinterpret_cast<int32_t*>(w + p.off_sorted);
    a.pair_pos = reinterpret_cast<int32_t*>(w + p.off_pos);
    a.tile_rec = reinterpret_cast<int4*>(w + p.off_tile);
    a.n_tiles = reinterpret_cast<int32_t*>(w + p.off_ntiles);
    a.chunk_count = reinterpret_cast<int32_t*>(w + p.off_chunk);
    a.n_chunks = p.n_chunks;
    a.hbuf = reinterpret_cast<uint16_t*>(w + p.off_h);
    a.ybuf = reinterpret_cast<float*>(w + p.off_y);
    a.error_word = reinterpret_cast<uint32_t*>(c->ws + c->err_off);
    a.pairs_cap = p.pairs_cap; a.tiles_cap = p.tiles_cap; a.m_tile = p.m_tile; a.ksplit = p.ksplit;
    a.tiled_waves = c->tune_tiled_waves;
    a.tiled_group = uint32_t(c->tune_tiled_group);
    a.tiled_persist = uint32_t(c->tune_tiled_persist);

    if (c->load_valid[layer]) HIPCHECK(hipStreamWaitEvent(stream, c->ev_load[layer], 0));
    if (c->rel_valid[layer]) HIPCHECK(hipStreamWaitEvent(stream, c->ev_rel[layer], 0));
    HIPCHECK(launch_ffn(a, c->n_cus, stream, c->profiling ? ffn_span_hook : nullptr, c));
    HIPCHECK(hipEventRecord(c->ev_infer[layer], stream));
    c->infer_valid[layer] = 1;
    const int64_t lo = int64_t(layer) * c->d.n_experts, hi = lo + c->d.n_experts;
    for (uint32_t s = 0; s < c->d.n_slots; ++s)
        if (c->slot_owner[s] >= lo && c->slot_owner[s] < hi) c->slot_last_reader[s] = int32_t(layer);
    return FLUXMOE_OK;
}

int fluxmoe_expert_ffn(fluxmoe_ctx* c, uint32_t layer, const uint16_t* tokens, uint32_t T,
                       const int32_t* topk_ids, const float* topk_w, uint32_t K,
                       const int32_t* page_table, float* out, uint32_t flags, void* stream_v) {
    if (int rc = check_layer(c, layer, false)) return rc;
    if (!c->arenas_bound) return set_error(FLUXMOE_ESTATE, "fluxmoe_bind_arenas has not been called");
    if (T == 0) return FLUXMOE_OK;
    return expert_ffn_enqueue(c, layer, tokens, T, topk_ids, topk_w, K, page_table, out, flags, stream_v,
                              c->ws + c->pool_ws_bytes, c->ws_bytes - c->pool_ws_bytes, "the bound workspace past the pool part");
}

int fluxmoe_expert_ffn_static(fluxmoe_ctx* c, uint32_t layer, const uint16_t* tokens, uint32_t T,
                              const int32_t* topk_ids, const float* topk_w, uint32_t K,
                              const int32_t* page_table, float* out, uint32_t flags, void* stream_v) {
    if (int rc = check_layer(c, layer, false)) return rc;
    if (!c->arenas_bound) return set_error(FLUXMOE_ESTATE, "fluxmoe_bind_arenas has not been called");
    if (T == 0) return FLUXMOE_OK;
    uint8_t* w = (c->device >= 0 && c->device < kMaxDevices) ? g_static_scratch[c->device] : nullptr;
    if (!w) return set_error(FLUXMOE_ESTATE, "the static scratch of device %d was not resolved at bind time", c->device);
    int dev = -1;
    HIPCHECK(hipGetDevice(&dev));
    if (dev != c->device)
        return set_error(FLUXMOE_ESTATE, "current device is %d, the context was bound on device %d", dev, c->device);
    return expert_ffn_enqueue(c, layer, tokens, T, topk_ids, topk_w, K, page_table, out, flags, stream_v,
                              w, kStaticScratchBytes, "the static FFN scratch");
}

int fluxmoe_shared_expert_ffn(fluxmoe_ctx* c, const uint16_t* w13, const uint16_t* w2,
                              const uint16_t* tokens, uint32_t T, float* out, uint32_t flags,
                              void* stream_v) {
    if (!c) return set_error(FLUXMOE_EINVAL, "ctx is NULL");
    if (!c->arenas_bound) return set_error(FLUXMOE_ESTATE, "fluxmoe_bind_arenas has not been called");
    if (T == 0) return FLUXMOE_OK;
    if (!w13 || !w2 || !tokens || !out) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if (flags & ~1u) return set_error(FLUXMOE_EINVAL, "only FLUXMOE_FFN_ACCUMULATE is accepted");
    if (T > 65535) return set_error(FLUXMOE_EINVAL, "T too large");
    if ((uintptr_t(w13) | uintptr_t(w2) | uintptr_t(tokens) | uintptr_t(out)) & 15)
        return set_error(FLUXMOE_EINVAL, "pointers must be 16-byte aligned");
    const FfnPlan p = plan_ffn(ffn_shape(c, 1), T, 1);   // this model's shapes, a single always-mapped expert
    const uint64_t extra = shared_extra_bytes(T);
    if (c->pool_ws_bytes + p.bytes + extra > c->ws_bytes)
        return set_error(FLUXMOE_ENOMEM, "workspace has %zu bytes, the shared expert with T=%u needs %llu",
                         c->ws_bytes, T, (unsigned long long)(c->pool_ws_bytes + p.bytes + extra));
    if (p.tiles_cap > 65535) return set_error(FLUXMOE_EINVAL, "too many row tiles (%u)", p.tiles_cap);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    uint8_t* w = c->ws + c->pool_ws_bytes;
    uint8_t* x = w + p.bytes;
    int32_t* ids = reinterpret_cast<int32_t*>(x);
    int32_t* gates = reinterpret_cast<int32_t*>(x + align_up(uint64_t(T) * 4, 256));
    int32_t* table = reinterpret_cast<int32_t*>(x + 2 * align_up(uint64_t(T) * 4, 256));
    HIPCHECK(launch_fill_i32(ids, 0, T, stream));
    HIPCHECK(launch_fill_i32(gates, 0x3F800000, T, stream));      // 1.0f
    HIPCHECK(launch_fill_i32(table, 0, 1, stream));
    FfnArgs a{};
    a.tokens = tokens;
    a.topk_ids = ids;
    a.topk_w = reinterpret_cast<const float*>(gates);
    a.page_table = table;
    a.slots13 = w13;
    a.slots2 = w2;
    a.out = out;
    a.T = T; a.K = 1; a.H = c->d.hidden; a.F = c->d.ffn; a.E = 1;
    a.flags = flags;
    a.expert_count = reinterpret_cast<int32_t*>(w + p.off_count);
    a.expert_offset = reinterpret_cast<int32_t*>(w + p.off_offset);
    a.sorted_pair = reinterpret_cast<int32_t*>(w + p.off_sorted);
    a.pair_pos = reinterpret_cast<int32_t*>(w + p.off_pos);
    a.tile_rec = reinterpret_cast<int4*>(w + p.off_tile);
    a.n_tiles = reinterpret_cast<int32_t*>(w + p.off_ntiles);
    a.chunk_count = reinterpret_cast<int32_t*>(w + p.off_chunk);
    a.n_chunks = p.n_chunks;
    a.hbuf = reinterpret_cast<uint16_t*>(w + p.off_h);
    a.ybuf = reinterpret_cast<float*>(w + p.off_y);
    a.error_word = reinterpret_cast<uint32_t*>(c->ws + c->err_off);
    a.pairs_cap = p.pairs_cap; a.tiles_cap = p.tiles_cap; a.m_tile = p.m_tile; a.ksplit = p.ksplit;
    a.tiled_waves = c->tune_tiled_waves;
    a.tiled_group = uint32_t(c->tune_tiled_group);
    a.tiled_persist = uint32_t(c->tune_tiled_persist);
    HIPCHECK(launch_ffn(a, c->n_cus, stream, c->profiling ? ffn_span_hook : nullptr, c));
    return FLUXMOE_OK;
}

int fluxmoe_stream_copy(void* dst, const void* src, uint64_t bytes, uint32_t n_workgroups, void* stream) {
    if (!dst || !src) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if ((uintptr_t(dst) | uintptr_t(src) | bytes) & 15) return set_error(FLUXMOE_EINVAL, "16-byte alignment required");
    if (n_workgroups == 0 || n_workgroups > (1u << 20)) return set_error(FLUXMOE_EINVAL, "bad n_workgroups");
    HIPCHECK(launch_stream_copy(dst, src, bytes, n_workgroups, static_cast<hipStream_t>(stream)));
    return FLUXMOE_OK;
}

int fluxmoe_stream_mix(void* dst, uint64_t dst_bytes, const void* src, uint64_t src_bytes, uint32_t out_bytes_small,
                       uint32_t waves_per_workgroup, uint32_t blocks_per_wave, uint32_t order, uint64_t* bytes_written,
                       void* stream) {
    if (!dst || !src) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if ((uintptr_t(dst) | uintptr_t(src)) & 127) return set_error(FLUXMOE_EINVAL, "128-byte alignment required");
    if (out_bytes_small < 128 || out_bytes_small > 16384 || out_bytes_small % 128)
        return set_error(FLUXMOE_EINVAL, "out_bytes_small must be a multiple of 128 in [128, 16384]");
    if (waves_per_workgroup != 4 && waves_per_workgroup != 8 && waves_per_workgroup != 16)
        return set_error(FLUXMOE_EINVAL, "waves_per_workgroup must be 4, 8 or 16");
    if (blocks_per_wave == 0 || blocks_per_wave > 1024) return set_error(FLUXMOE_EINVAL, "bad blocks_per_wave");
    if (order > 2) return set_error(FLUXMOE_EINVAL, "order must be 0, 1 or 2");
    const uint64_t n_blocks = src_bytes / 4096;
    if (n_blocks == 0 || n_blocks > (1ull << 30)) return set_error(FLUXMOE_EINVAL, "src must hold 1 to 2^30 blocks of 4096 bytes");
    const uint64_t need = stream_mix_out_bytes(n_blocks, out_bytes_small);
    if (dst_bytes < need)
        return set_error(FLUXMOE_EINVAL, "dst holds %llu bytes, %llu blocks write %llu", (unsigned long long)dst_bytes,
                         (unsigned long long)n_blocks, (unsigned long long)need);
    const uint64_t per_wg = uint64_t(waves_per_workgroup) * blocks_per_wave;
    const uint64_t n_wg = (n_blocks + per_wg - 1) / per_wg;
    if (n_wg > (1u << 24)) return set_error(FLUXMOE_EINVAL, "too many workgroups (%llu)", (unsigned long long)n_wg);
    HIPCHECK(launch_stream_mix(dst, src, uint32_t(n_blocks), out_bytes_small, int(waves_per_workgroup), blocks_per_wave,
                               order, uint32_t(n_wg), static_cast<hipStream_t>(stream)));
    if (bytes_written) *bytes_written = need;
    return FLUXMOE_OK;
}

int fluxmoe_mfma_probe(const void* operands, float* out, uint32_t n_workgroups, uint32_t iters, void* stream) {
    if (!operands || !out) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if ((uintptr_t(operands) & 15) || (uintptr_t(out) & 3)) return set_error(FLUXMOE_EINVAL, "operands must be 16-byte aligned");
    if (n_workgroups == 0 || n_workgroups > (1u << 16) || iters == 0) return set_error(FLUXMOE_EINVAL, "bad n_workgroups or iters");
    HIPCHECK(launch_mfma_probe(operands, out, n_workgroups, iters, static_cast<hipStream_t>(stream)));
    return FLUXMOE_OK;
}

int fluxmoe_profile_enable(fluxmoe_ctx* c, int on) {
    if (!c) return set_error(FLUXMOE_EINVAL, "ctx is NULL");
    c->profiling = on != 0;
    c->profile_mask = (on & 0x100) ? uint32_t(on & 0x1F) : 0x1Fu;
    return FLUXMOE_OK;
}

int fluxmoe_profile_collect(fluxmoe_ctx* c, double out_ms[FLUXMOE_PROFILE_KINDS],
                            uint32_t out_count[FLUXMOE_PROFILE_KINDS]) {
    if (!c || !out_ms || !out_count) return set_error(FLUXMOE_EINVAL, "NULL argument");
    for (int k = 0; k < FLUXMOE_PROFILE_KINDS; ++k) { out_ms[k] = 0; out_count[k] = 0; }
    for (auto& sp : c->spans) {
        HIPCHECK(hipEventSynchronize(sp.b));
        float ms = 0;
        HIPCHECK(hipEventElapsedTime(&ms, sp.a, sp.b));
        out_ms[sp.kind] += ms;
        out_count[sp.kind] += 1;
        (void)hipEventDestroy(sp.a);
        (void)hipEventDestroy(sp.b);
    }
    c->spans.clear();
    return FLUXMOE_OK;
}

int fluxmoe_device_errors(fluxmoe_ctx* c, uint32_t* out_flags) {
    if (!c || !out_flags) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if (!c->arenas_bound) return set_error(FLUXMOE_ESTATE, "fluxmoe_bind_arenas has not been called");
    HIPCHECK(hipDeviceSynchronize());
    HIPCHECK(hipMemcpy(out_flags, c->ws + c->err_off, 4, hipMemcpyDeviceToHost));
    HIPCHECK(hipMemset(c->ws + c->err_off, 0, 4));
    return FLUXMOE_OK;
}

}  // extern "C"
