// Routed SwiGLU expert FFN over page-table addressed slots (gfx950, BF16 MFMA, FP32 acc).
//
// The paper runs an unchanged fused-MoE kernel on the materialized tensors (Sec. 5; tensor
// types of Sec. 4.1 "Formal model": fused gate/up [2][H][F] and down [F][H]); it gives no
// kernel design, so this one is built for decode-shaped batches on MI355X, where every
// expert sees few tokens and the FFN is bound by streaming the expert's weights once:
//
//   route_sort   one workgroup: counting sort of the (token, k) pairs by expert, skipping
//                pairs whose expert has no slot; emits one record per row tile (expert, first
//                row, rows, slot), tiles with the most rows first
//   gemm1        per (row tile, 128-column strip): a = X W1 and b = X W3 on two wavefronts
//                with v_mfma_f32_16x16x32_bf16, h = silu(a) * b rounded to BF16
//   gemm2        per (row tile, 128-column strip, K split): y = h W2, FP32 partial sums
//   combine      out[t] = sum_k gate[t][k] * sum_splits y[pos(t,k)]   (fixed order)
//
// Weights stay row-major [K][N] in the slots (placement is bit-exact by contract), while
// MFMA wants 8 consecutive k per lane.  Each lane therefore loads 8 rows x 16 bytes (8
// columns) straight from HBM, fully coalesced along N, and transposes its 8x8 tile in
// registers with v_perm_b32; MFMA number c of a step uses column c of every lane's tile,
// so output column j of that MFMA is column 8 * j + c of the strip.  Weights never pass
// through LDS and every weight byte is read exactly once per row tile; LDS holds only the
// tile's activations, shared by the four wavefronts of a workgroup.
// Batches with more rows per expert than one 128-row tile go to the LDS-tiled kernels
// further down (gemm_d2l_kernel and its register-staged predecessors), which are bound by
// the matrix cores.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "kernels.h"

namespace fluxmoe {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

union Frag {
    uint4 u;
    bf16x8 v;
};

constexpr int kStrip = 128;        // output columns per wavefront
constexpr int kChunk = 32;         // k per MFMA step
constexpr int kNonTemporal = 2;    // cache policy operand of the buffer loads: bit 1 = nt

// ------------------------------------------------------------------ routing / grouping
// Row tiles are handed out by size class: the body a tile runs and the time it takes grow with its rows,
// and a launch ends when its last workgroup does, so the tiles with the most rows are numbered (and
// therefore started) first and the many small ones fill in behind them.
constexpr int kTileClasses = 5;
__device__ __forceinline__ int tile_class(int32_t rows) {
    return rows > 96 ? 0 : (rows > 64 ? 1 : (rows > 32 ? 2 : (rows > 16 ? 3 : 4)));
}

// Exclusive prefix sums over the 1024 threads of a workgroup for N values per thread at once; total[i]
// receives the sum of v[i] over all threads.  tot: N * 17 ints of LDS.  Contains barriers.
template <int N>
__device__ __forceinline__ void block_scan_excl(const int32_t (&v)[N], int32_t (&excl)[N], int32_t (&total)[N], int32_t* tot) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t x[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        x[i] = v[i];
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int32_t y = __shfl_up(x[i], d, 64);
            if (lane >= d) x[i] += y;
        }
        if (lane == 63) tot[i * 17 + wave] = x[i];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int32_t w = lane < 16 ? tot[i * 17 + lane] : 0;
            int32_t xs = w;
#pragma unroll
            for (int d = 1; d < 16; d <<= 1) {
                const int32_t y = __shfl_up(xs, d, 64);
                if (lane >= d) xs += y;
            }
            if (lane < 16) tot[i * 17 + lane] = xs - w;
            if (lane == 15) tot[i * 17 + 16] = xs;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < N; ++i) {
        excl[i] = x[i] - v[i] + tot[i * 17 + wave];
        total[i] = tot[i * 17 + 16];
    }
    __syncthreads();
}

// Large batches: one workgroup per chunk of kRouteChunkPairs pairs counts its pairs per expert
// (route_count_kernel), the single workgroup of route_sort_kernel<true> adds the chunks up, turns each
// chunk's count into the chunk's first position inside the expert's rows and does the scans and the tile
// records, and one workgroup per chunk puts its pairs in place (route_scatter_kernel).  The positions a
// chunk's pairs get depend only on the chunk, not on which workgroup runs first.
__device__ __forceinline__ int32_t route_classify(const FfnArgs& a, int32_t e, const int32_t* slot_of, bool report) {
    if (e < 0 || uint32_t(e) >= a.E) {
        if (report) atomicOr(a.error_word, 2u);
        return -1;
    }
    if (slot_of[e] < 0) {
        if (report && !(a.flags & 2u)) atomicOr(a.error_word, 2u);
        return -1;
    }
    return e;
}

__global__ __launch_bounds__(1024) void route_count_kernel(FfnArgs a) {
    extern __shared__ int32_t sh[];          // count[E]
    const uint32_t pairs = a.T * a.K, first = blockIdx.x * kRouteChunkPairs;
    for (uint32_t e = threadIdx.x; e < a.E; e += 1024) sh[e] = 0;
    __syncthreads();
    for (uint32_t p = first + threadIdx.x; p < min(pairs, first + kRouteChunkPairs); p += 1024) {
        const int32_t e = route_classify(a, a.topk_ids[p], a.page_table, true);
        if (e >= 0) atomicAdd(&sh[e], 1);
    }
    __syncthreads();
    for (uint32_t e = threadIdx.x; e < a.E; e += 1024) a.chunk_count[size_t(blockIdx.x) * a.E + e] = sh[e];
}

__global__ __launch_bounds__(1024) void route_scatter_kernel(FfnArgs a) {
    extern __shared__ int32_t sh[];          // cursor[E]
    const uint32_t pairs = a.T * a.K, first = blockIdx.x * kRouteChunkPairs;
    for (uint32_t e = threadIdx.x; e < a.E; e += 1024) sh[e] = a.expert_offset[e] + a.chunk_count[size_t(blockIdx.x) * a.E + e];
    __syncthreads();
    for (uint32_t p = first + threadIdx.x; p < min(pairs, first + kRouteChunkPairs); p += 1024) {
        const int32_t e = route_classify(a, a.topk_ids[p], a.page_table, false);
        int32_t pos = -1;
        if (e >= 0) {
            pos = atomicAdd(&sh[e], 1);
            a.sorted_pair[pos] = int32_t(p);
        }
        a.pair_pos[p] = pos;
    }
}

template <bool CHUNKED>
__global__ __launch_bounds__(1024) void route_sort_kernel(FfnArgs a) {
    extern __shared__ int32_t sh[];          // count[E], cursor[E], slot[E], scan scratch
    int32_t* count = sh;
    int32_t* cursor = sh + a.E;
    int32_t* slot_of = sh + 2 * a.E;         // this layer's page-table row: every later look-up is an LDS read
    int32_t* scratch = sh + 3 * a.E;
    __shared__ int32_t class_total[kTileClasses];
    const int tid = threadIdx.x;
    const uint32_t pairs = a.T * a.K;
    const int32_t m = int32_t(a.m_tile);
    for (uint32_t e = tid; e < a.E; e += 1024) { count[e] = 0; slot_of[e] = a.page_table[e]; }
    if (tid < kTileClasses) class_total[tid] = 0;
    // the first pairs' expert ids are fetched while the page-table row is on its way
    constexpr int kKept = 8;
    int32_t kept[kKept];
#pragma unroll
    for (int i = 0; i < kKept; ++i) {
        const uint32_t p = tid + 1024u * i;
        kept[i] = (!CHUNKED && p < pairs) ? a.topk_ids[p] : -1;
    }
    if (CHUNKED) {
        // the chunks' counts, added up per expert; each is replaced by the sum of the chunks before it
        for (uint32_t e = tid; e < a.E; e += 1024) {
            int32_t run = 0;
            for (uint32_t c = 0; c < a.n_chunks; ++c) {
                const int32_t v = a.chunk_count[size_t(c) * a.E + e];
                a.chunk_count[size_t(c) * a.E + e] = run;
                run += v;
            }
            count[e] = run;
        }
    }
    __syncthreads();
    // a thread's first kKept pairs stay in registers for the scatter at the end (expert, or -1 for a pair
    // that is skipped); batches with more pairs per thread read the rest again
    auto classify = [&](int32_t e, bool report) { return route_classify(a, e, slot_of, report); };
    if (!CHUNKED) {
#pragma unroll
        for (int i = 0; i < kKept; ++i) {
            const uint32_t p = tid + 1024u * i;
            kept[i] = p < pairs ? classify(kept[i], true) : -1;
            if (kept[i] >= 0) atomicAdd(&count[kept[i]], 1);
        }
        for (uint32_t p = tid + 1024u * kKept; p < pairs; p += 1024) {
            const int32_t e = classify(a.topk_ids[p], true);
            if (e >= 0) atomicAdd(&count[e], 1);
        }
    }
    __syncthreads();
    // Tiles per class over all experts, needed before the tiles of the first 1024 experts can be numbered.  With one
    // round (at most 1024 experts) the round's own scan delivers them; otherwise they are summed here
    // (integer sums: the order of the additions does not matter).
    const bool one_round = a.E <= 1024;
    if (!one_round) {
        for (uint32_t e = tid; e < a.E; e += 1024) {
            const int32_t c = count[e];
            if (c >= m) atomicAdd(&class_total[tile_class(m)], c / m);
            if (c % m) atomicAdd(&class_total[tile_class(c % m)], 1);
        }
        __syncthreads();
    }
    int32_t class_base[kTileClasses];        // first tile number of each class; advanced round by round
    int32_t n_tiles = 0;
#pragma unroll
    for (int k = 0; k < kTileClasses; ++k) { class_base[k] = n_tiles; n_tiles += class_total[k]; }
    int32_t row_base = 0;
    // experts in rounds of 1024, one per thread: exclusive scans of its rows and of its tiles in each class
    for (uint32_t base = 0; base < a.E; base += 1024) {
        const uint32_t e = base + tid;
        const int32_t c = (e < a.E) ? count[e] : 0;
        const int32_t full = c / m, rem = c % m;
        const int k_full = tile_class(m), k_rem = tile_class(rem);
        int32_t v[1 + kTileClasses], excl[1 + kTileClasses], total[1 + kTileClasses];
        v[0] = c;
#pragma unroll
        for (int k = 0; k < kTileClasses; ++k) v[1 + k] = (k == k_full ? full : 0) + ((rem && k == k_rem) ? 1 : 0);
        block_scan_excl(v, excl, total, scratch);
        if (one_round) {
            n_tiles = 0;
#pragma unroll
            for (int k = 0; k < kTileClasses; ++k) { class_base[k] = n_tiles; n_tiles += total[1 + k]; }
        }
        if (e < a.E) {
            const int32_t row_excl = row_base + excl[0];
            a.expert_offset[e] = row_excl;
            a.expert_count[e] = c;
            cursor[e] = row_excl;
            const int32_t slot = c ? slot_of[e] : -1;
            int32_t at_full = 0, at_rem = 0;
#pragma unroll
            for (int k = 0; k < kTileClasses; ++k) {
                if (k == k_full) at_full = class_base[k] + excl[1 + k];
                if (k == k_rem) at_rem = class_base[k] + excl[1 + k] + (k == k_full ? full : 0);
            }
            for (int32_t i = 0; i < full; ++i)
                if (uint32_t(at_full + i) < a.tiles_cap) a.tile_rec[at_full + i] = make_int4(int32_t(e), row_excl + i * m, m, slot);
            if (rem && uint32_t(at_rem) < a.tiles_cap) a.tile_rec[at_rem] = make_int4(int32_t(e), row_excl + full * m, rem, slot);
        }
        row_base += total[0];
#pragma unroll
        for (int k = 0; k < kTileClasses; ++k) class_base[k] += total[1 + k];
    }
    // the records past the last tile read as empty tiles
    for (uint32_t i = uint32_t(min(n_tiles, int32_t(a.tiles_cap))) + tid; i < a.tiles_cap; i += 1024) a.tile_rec[i] = make_int4(0, 0, 0, -1);
    if (tid == 0) {
        a.expert_offset[a.E] = row_base;
        a.n_tiles[0] = min(n_tiles, int32_t(a.tiles_cap));
    }
    if (CHUNKED) return;                     // route_scatter_kernel puts the pairs in place
    __syncthreads();
    auto place = [&](uint32_t p, int32_t e) {
        int32_t pos = -1;
        if (e >= 0) {
            pos = atomicAdd(&cursor[e], 1);
            a.sorted_pair[pos] = int32_t(p);
        }
        a.pair_pos[p] = pos;
    };
#pragma unroll
    for (int i = 0; i < kKept; ++i) {
        const uint32_t p = tid + 1024u * i;
        if (p < pairs) place(p, kept[i]);
    }
    for (uint32_t p = tid + 1024u * kKept; p < pairs; p += 1024) place(p, classify(a.topk_ids[p], false));
}

// SiLU(g) * u (Sec. 2.1's gated FFN) in FP32 with the hardware's exp2 and reciprocal, each within one
// ulp; the caller rounds the product to BF16.  g -> -inf gives exp2 = +inf, reciprocal 0, product -0.
__device__ __forceinline__ float swiglu(float g, float u) {
    const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * g);
    return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

// ------------------------------------------------------------------ strip GEMM core
__device__ __forceinline__ uint32_t comp(const uint4& v, int i) {
    return i == 0 ? v.x : (i == 1 ? v.y : (i == 2 ? v.z : v.w));
}

// k chunks per wavefront held in the register ring (one being multiplied, the rest in flight)
template <int MI> struct RingDepth { static constexpr int value = MI >= 8 ? 2 : (MI >= 4 ? 3 : 4); };

// Shared A blocks: the four wavefronts of a workgroup multiply the same rows of A, so a block of
// kABlock k values of the tile's rows is loaded once per workgroup into LDS (two buffers) instead of
// once per wavefront from L2 (where it costs 0.75 bytes of requests per weight byte streamed).
constexpr int kABlock = 128;                 // k per block = 4 chunks

// acc += a * b (v_mfma_f32_16x16x32_bf16) with the accumulator pinned to the AGPR half of the register
// file.  Written as assembly because with the builtin the register allocator, short of VGPRs for
// 192 accumulators plus the load ring, parks ring registers in AGPRs and moves them back (more
// v_accvgpr moves than MFMAs in the ring loop).  The matrix-core hazards the compiler would cover
// are covered here: s_nop 1 gives the two wait states between a VALU write of an operand (the
// v_perm transposes, the v_accvgpr_write zeroing) and the MFMA that reads it; mfma_drain() must
// run before anything but another mfma16 reads an accumulator.  volatile keeps the statements in
// program order (loads and LDS reads stay where the source puts them relative to the MFMAs).
__device__ __forceinline__ void mfma16(f32x4& acc, const bf16x8& a, const bf16x8& b) {
    asm volatile("s_nop 1\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// 2 x 16 wait states: more than the 18 the longest matrix instruction needs before its result may
// be read by a vector, memory or LDS instruction
__device__ __forceinline__ void mfma_drain() {
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}

// One wavefront's product C[16*MI rows][128 columns] = A[rows][k range] * B[k range][strip].
template <int MI>
struct StripGemm {
    f32x4 acc[MI][8];

    static constexpr int kABufElems = 16 * MI * kABlock;     // one LDS buffer (rows of 256 bytes)

    // B rows come through buffer loads: one descriptor per expert matrix (scalar registers), one
    // VGPR with the lane's byte offset inside a chunk, and the row's byte offset as the scalar
    // offset operand - no vector arithmetic per load.  row0_bytes: offset of the chunk's first row.
    // The loads carry the non-temporal hint (cache policy bit 1): a decode-shaped batch reads every
    // weight byte once, and without the hint the stream pushes the activations, h and the partial
    // sums out of the caches (measured: 6 to 10 % more weight bytes per second with it).
    __device__ __forceinline__ static void load_b(uint4 (&b)[8], __amdgpu_buffer_rsrc_t rsrc, uint32_t voff,
                                                  uint32_t row0_bytes, uint32_t row_bytes) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, row0_bytes + uint32_t(r) * row_bytes, kNonTemporal);
            b[r] = make_uint4(v.x, v.y, v.z, v.w);
        }
    }

    __device__ __forceinline__ void mma_b(const uint4 (&b)[8], const uint4 (&a)[MI]) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            Frag f;
            const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
            f.u.x = __builtin_amdgcn_perm(comp(b[1], c >> 1), comp(b[0], c >> 1), sel);
            f.u.y = __builtin_amdgcn_perm(comp(b[3], c >> 1), comp(b[2], c >> 1), sel);
            f.u.z = __builtin_amdgcn_perm(comp(b[5], c >> 1), comp(b[4], c >> 1), sel);
            f.u.w = __builtin_amdgcn_perm(comp(b[7], c >> 1), comp(b[6], c >> 1), sel);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                Frag fa;
                fa.u = a[mi];
                mfma16(acc[mi][c], fa.v, f.v);
            }
        }
    }

    // The first n_blocks * kABlock k values of the range with A shared through LDS.  Every wavefront
    // of the four in the workgroup must call this with the same abase, k_begin and n_blocks (it
    // contains barriers).
    // A: a block is 16 MI rows x 128 k; it goes from global memory straight into LDS
    // (global_load_lds_dwordx4: no registers, no LDS write instructions), one instruction per
    // wavefront per 16 rows: lane (tid / 16, tid % 16) brings one 16-byte piece of row 16 i + tid / 16.
    // Such a load fills 1 KiB contiguously, so rows are 256 bytes apart with no padding; to keep the
    // 16-byte fragment reads of 16 consecutive rows on different banks, position p of row r holds
    // piece p ^ (r % 16).  abase is uniform over the workgroup; aoff[i] is the thread's byte offset of
    // piece (tid % 16) ^ (tid / 16 % 16) of row 16 i + tid / 16 (clamped to the tile's last row).
    // B: bmat points at the [k_rows][ldb] matrix (uniform over the wavefront, under 4 GiB), col is the
    // lane's first column; a four-deep register ring as in run().
    __device__ __forceinline__ void run_shared(const uint8_t* abase, const uint32_t (&aoff)[MI], uint16_t* abuf,
                                               const uint16_t* bmat, uint32_t k_rows, uint32_t col, uint32_t ldb,
                                               uint32_t k_begin, uint32_t n_blocks, int lane, int wave) {
        if (n_blocks == 0) return;
        const uint32_t kg = 8u * (uint32_t(lane) >> 4);
        const uint32_t row_bytes = 2u * ldb;
        // descriptor word 3 = 0x00020000: raw 32-bit data format of this architecture family
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t*>(bmat), 0, int(k_rows * row_bytes), 0x00020000);
        const uint32_t voff = kg * row_bytes + 2u * col;
        const uint32_t first_bytes = k_begin * row_bytes;
        const uint32_t chunk_bytes = uint32_t(kChunk) * row_bytes;
        // fragment of chunk c, tile mi: row 16 mi + lane % 16, piece 4 c + lane / 16
        const int a_fr = (lane & 15) * (2 * kABlock) + 16 * ((lane >> 4) ^ (lane & 15));   // bytes; ^ 64 c, + 4096 mi
        const uint8_t* const abuf8 = reinterpret_cast<const uint8_t*>(abuf);
        const uint32_t abuf_lds = uint32_t(uintptr_t((__attribute__((address_space(3))) void*)abuf));
        uint4 bst[4][8];
        // M0 carries the LDS destination of an LDS-direct load and is read when the instruction
        // issues; the compiler reserves it, so its value is put back
        auto a_dma = [&](uint32_t blk, uint32_t buf_bytes) __attribute__((always_inline)) {
            const uint8_t* src = abase + (size_t(k_begin) + size_t(blk) * kABlock) * 2;
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                uint32_t saved_m0;
                const uint32_t dst = abuf_lds + buf_bytes + uint32_t(i * 4 + wave) * 1024u;
                asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
                             : "=&s"(saved_m0) : "v"(aoff[i]), "s"(src), "s"(dst) : "memory");
            }
        };
        constexpr uint32_t kBufBytes = uint32_t(kABufElems) * 2;
        // one block of four chunks; PREFETCH: all four B loads three chunks ahead are inside the
        // shared range and the next A block exists
        auto block = [&](uint32_t cur_bytes, uint32_t nxt_bytes, uint32_t blk, auto PREFETCH) __attribute__((always_inline)) {
            if (PREFETCH.value) a_dma(blk + 1, nxt_bytes);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t chunk = blk * 4 + c;
                if (PREFETCH.value || chunk + 3 < n_blocks * 4) load_b(bst[(c + 3) & 3], rsrc, voff, first_bytes + (chunk + 3) * chunk_bytes, row_bytes);
                uint4 af[MI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    af[mi] = *reinterpret_cast<const uint4*>(abuf8 + cur_bytes + ((a_fr ^ (64 * c)) + 4096 * mi));
                mma_b(bst[c], af);
            }
            // the A block fetched above was issued before this block's 32 B loads and loads return in
            // order: at most the 24 newest (three chunks of B) may still be in flight
            if (PREFETCH.value) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
            __syncthreads();
        };
        a_dma(0, 0);
#pragma unroll
        for (int c = 0; c < 3; ++c) load_b(bst[c], rsrc, voff, first_bytes + uint32_t(c) * chunk_bytes, row_bytes);
        asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
        __syncthreads();
        uint32_t blk = 0;
        for (; blk + 1 < n_blocks; ++blk)
            block((blk & 1) * kBufBytes, ((blk + 1) & 1) * kBufBytes, blk, std::integral_constant<bool, true>{});
        block((blk & 1) * kBufBytes, ((blk + 1) & 1) * kBufBytes, blk, std::integral_constant<bool, false>{});
        mfma_drain();
    }

    struct Stage {
        uint4 b[8];      // the lane's 8 rows x 8 columns of B
        uint4 a[MI];     // the lane's A fragments (8 consecutive k of one row per 16-row tile)
    };

    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[mi][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    __device__ __forceinline__ static void load(Stage& st, const uint16_t* const (&arow)[MI],
                                                const uint16_t* bcol, size_t ldb, uint32_t k0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) st.b[r] = load_stream16(bcol + size_t(k0 + r) * ldb);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) st.a[mi] = *reinterpret_cast<const uint4*>(arow[mi] + k0);
    }

    __device__ __forceinline__ void mma(const Stage& st) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            Frag f;
            const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
            f.u.x = __builtin_amdgcn_perm(comp(st.b[1], c >> 1), comp(st.b[0], c >> 1), sel);
            f.u.y = __builtin_amdgcn_perm(comp(st.b[3], c >> 1), comp(st.b[2], c >> 1), sel);
            f.u.z = __builtin_amdgcn_perm(comp(st.b[5], c >> 1), comp(st.b[4], c >> 1), sel);
            f.u.w = __builtin_amdgcn_perm(comp(st.b[7], c >> 1), comp(st.b[6], c >> 1), sel);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                Frag fa;
                fa.u = st.a[mi];
                mfma16(acc[mi][c], fa.v, f.v);
            }
        }
    }

    // k range a multiple of 8.  bcol must point at 8 existing columns for every lane (callers
    // clamp lanes past the edge).  A ring of 3-4 register stages keeps all but one chunk
    // of 32 k in flight while that one is multiplied: with one wavefront per SIMD that is what
    // covers HBM latency.  A k range that is not a multiple of 32 ends with one chunk in
    // which the lanes past the end contribute zeros.
    __device__ __forceinline__ void run(const uint16_t* const (&arow)[MI], const uint16_t* bcol,
                                        size_t ldb, uint32_t k_begin, uint32_t k_end, int lane) {
        constexpr int kStages = RingDepth<MI>::value;
        if (k_begin >= k_end) return;
        const uint32_t kg = 8u * (uint32_t(lane) >> 4);
        const uint32_t n = (k_end - k_begin) / kChunk;
        const uint32_t kb = k_begin + kg;
        Stage st[kStages];
#pragma unroll
        for (int s = 0; s < kStages - 1; ++s)
            if (uint32_t(s) < n) load(st[s], arow, bcol, ldb, kb + s * kChunk);
        // Steady state without branches: a conditional load inside the loop makes the compiler
        // wait for the newest loads at the join (it must assume the path that issued none), which
        // serialises the ring.  Rounds in which every load is in range run unconditionally; the
        // last rounds take the guarded form.
        uint32_t base = 0;
        for (; base + 2 * kStages - 2 < n; base += kStages) {
#pragma unroll
            for (int s = 0; s < kStages; ++s) {
                load(st[(s + kStages - 1) % kStages], arow, bcol, ldb, kb + (base + s + kStages - 1) * kChunk);
                mma(st[s]);
            }
        }
        for (; base < n; base += kStages) {
#pragma unroll
            for (int s = 0; s < kStages; ++s) {
                const uint32_t i = base + s;
                if (i < n) {
                    if (i + kStages - 1 < n)
                        load(st[(s + kStages - 1) % kStages], arow, bcol, ldb, kb + (i + kStages - 1) * kChunk);
                    mma(st[s]);
                }
            }
        }
        const uint32_t k_full = k_begin + n * kChunk;
        if (k_full < k_end) {
            const uint4 z = make_uint4(0, 0, 0, 0);
            Stage t;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) t.a[mi] = z;
#pragma unroll
            for (int r = 0; r < 8; ++r) t.b[r] = z;
            if (k_full + kg < k_end) load(t, arow, bcol, ldb, k_full + kg);
            mma(t);
        }
        mfma_drain();
    }
};

// Two FP32 values rounded to BF16 (nearest even) and packed, lo in bits 0..15: one v_cvt_pk_bf16_f32.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

struct TileInfo {
    int32_t expert, row0, rows, slot;
};

// One 16-byte load: route_sort_kernel wrote (expert, first row, rows, slot) for every tile number below
// tiles_cap, with rows = 0 past the last tile.
__device__ __forceinline__ bool tile_info(const FfnArgs& a, uint32_t tile, TileInfo& t) {
    const int4 r = a.tile_rec[tile];
    t.expert = r.x; t.row0 = r.y; t.rows = r.z; t.slot = r.w;
    return t.rows > 0 && t.slot >= 0;
}

// h[row][n] = bf16( silu(x W1) * (x W3) ).  A workgroup is two pairs of wavefronts; each
// pair owns one 128-column strip: the even wavefront multiplies by W1 (gate), the odd one by
// W3 (up), the odd one hands its accumulators over through LDS and the even one applies
// SwiGLU and stores.  Splitting the two matrices over two wavefronts halves the accumulator
// registers per wavefront, which is what leaves room for the deep load ring.
template <int MI>
__device__ __forceinline__ void gemm1_swiglu_body(const FfnArgs& a, const TileInfo& t, float (*xch)[64], uint16_t* abuf) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6));   // uniform: scalar address arithmetic
    const int pair = wave >> 1;
    const int mat_id = wave & 1;
    const uint32_t strip = blockIdx.x * 2 + pair;
    const uint32_t n0 = strip * kStrip + 8u * (lane & 15);
    const bool col_ok = n0 < a.F;                 // strips past F still run (barrier below)

    const uint16_t* arow[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int32_t r = min(mi * 16 + (lane & 15), t.rows - 1);
        const int32_t pr = a.sorted_pair[t.row0 + r];
        const uint32_t tok = uint32_t(pr) / a.K;
        arow[mi] = a.tokens + size_t(tok) * a.H;
    }
    const size_t mat = size_t(a.H) * a.F;
    const uint16_t* w = a.slots13 + size_t(t.slot) * 2 * mat + size_t(mat_id) * mat;

    // the thread's pieces of the shared A blocks: row 16 i + tid / 16, piece (tid % 16) ^ (tid / 16 % 16)
    const uint32_t piece = (threadIdx.x & 15u) ^ ((threadIdx.x >> 4) & 15u);
    uint32_t aoff[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int32_t r = min(i * 16 + int(threadIdx.x >> 4), t.rows - 1);
        const int32_t pr = a.sorted_pair[t.row0 + r];
        aoff[i] = 2u * ((uint32_t(pr) / a.K) * a.H + 8u * piece);          // the launcher checks T * H * 2 < 4 GiB
    }
    StripGemm<MI> g;
    g.zero();
    const uint32_t n_blocks = a.H / kABlock;
    g.run_shared(reinterpret_cast<const uint8_t*>(a.tokens), aoff, abuf, w, a.H, col_ok ? n0 : a.F - 8, a.F, 0, n_blocks, lane, wave);
    g.run(arow, w + (col_ok ? n0 : a.F - 8), a.F, n_blocks * kABlock, a.H, lane);

    if (mat_id == 1) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int c = 0; c < 8; ++c)
#pragma unroll
                for (int r = 0; r < 4; ++r) xch[pair * (MI * 32) + (mi * 8 + c) * 4 + r][lane] = g.acc[mi][c][r];
    }
    __syncthreads();
    if (mat_id == 1 || !col_ok) return;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int32_t row = mi * 16 + 4 * (lane >> 4) + r;
            if (row >= t.rows) continue;
            float hv[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const float ga = g.acc[mi][c][r];
                const float up = xch[pair * (MI * 32) + (mi * 8 + c) * 4 + r][lane];
                hv[c] = swiglu(ga, up);
            }
            uint4 o;
            o.x = pack_bf16_rne(hv[0], hv[1]);
            o.y = pack_bf16_rne(hv[2], hv[3]);
            o.z = pack_bf16_rne(hv[4], hv[5]);
            o.w = pack_bf16_rne(hv[6], hv[7]);
            *reinterpret_cast<uint4*>(a.hbuf + size_t(t.row0 + row) * a.F + n0) = o;
        }
}

// Row tiles hold up to 16 MI rows so that an expert's weights are streamed once even when routing is
// skewed (an expert with 231 of 2560 pairs next to hundreds with five); a tile with fewer rows takes a
// body compiled for fewer 16-row MFMA tiles (less matrix work per chunk, same registers reserved).
template <int MI>
__global__ __launch_bounds__(256) void gemm1_swiglu_kernel(FfnArgs a) {
    // the accumulator exchange of the epilogue ([pair][mi, c, r][lane] floats) reuses the memory of
    // the shared A blocks: every wavefront has passed the last block's barrier by then
    constexpr size_t kXchBytes = sizeof(float) * 2 * MI * 8 * 4 * 64;
    constexpr size_t kABytes = sizeof(uint16_t) * 2 * StripGemm<MI>::kABufElems;
    __shared__ __align__(16) uint8_t smem[kXchBytes > kABytes ? kXchBytes : kABytes];
    float (*xch)[64] = reinterpret_cast<float (*)[64]>(smem);
    uint16_t* abuf = reinterpret_cast<uint16_t*>(smem);
    TileInfo t;
    if (!tile_info(a, blockIdx.y, t)) return;     // uniform over the workgroup
    if (MI > 1 && t.rows <= 16) gemm1_swiglu_body<1>(a, t, xch, abuf);
    else if (MI > 2 && t.rows <= 32) gemm1_swiglu_body<2>(a, t, xch, abuf);
    else if (MI > 4 && t.rows <= 64) gemm1_swiglu_body<4>(a, t, xch, abuf);
    else if (MI > 6 && t.rows <= 96) gemm1_swiglu_body<6>(a, t, xch, abuf);
    else gemm1_swiglu_body<MI>(a, t, xch, abuf);
}

// y[split][row][n] = h[row][k range] W2[k range][n]
template <int MI>
__device__ __forceinline__ void gemm2_body(const FfnArgs& a, const TileInfo& t, uint16_t* abuf, uint32_t col_wg, uint32_t split) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6));
    const uint32_t strip = col_wg * 4 + wave;
    const uint32_t n0 = strip * kStrip + 8u * (lane & 15);
    const bool col_ok = n0 < a.H;                 // wavefronts past the last strip still run (barriers below)
    const uint32_t k_per = ((a.F + a.ksplit - 1) / a.ksplit + kChunk - 1) / kChunk * kChunk;
    const uint32_t k_begin = min(a.F, split * k_per);
    const uint32_t k_end = min(a.F, k_begin + k_per);

    const uint16_t* arow[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int32_t r = min(mi * 16 + (lane & 15), t.rows - 1);
        arow[mi] = a.hbuf + size_t(t.row0 + r) * a.F;
    }
    const uint16_t* w2 = a.slots2 + size_t(t.slot) * a.F * a.H;

    // the thread's pieces of the shared A blocks, as byte offsets from the tile's first row of h
    const uint32_t piece = (threadIdx.x & 15u) ^ ((threadIdx.x >> 4) & 15u);
    uint32_t aoff[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int32_t r = min(i * 16 + int(threadIdx.x >> 4), t.rows - 1);
        aoff[i] = 2u * (uint32_t(r) * a.F + 8u * piece);
    }
    StripGemm<MI> g;
    g.zero();
    const uint32_t n_blocks = (k_end - k_begin) / kABlock;
    g.run_shared(reinterpret_cast<const uint8_t*>(a.hbuf + size_t(t.row0) * a.F), aoff, abuf, w2, a.F, col_ok ? n0 : a.H - 8, a.H,
                 k_begin, n_blocks, lane, wave);
    g.run(arow, w2 + (col_ok ? n0 : a.H - 8), a.H, k_begin + n_blocks * kABlock, k_end, lane);

    if (!col_ok) return;
    float* y = a.ybuf + size_t(split) * a.pairs_cap * a.H;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int32_t row = mi * 16 + 4 * (lane >> 4) + r;
            if (row >= t.rows) continue;
            float4 lo = make_float4(g.acc[mi][0][r], g.acc[mi][1][r], g.acc[mi][2][r], g.acc[mi][3][r]);
            float4 hi = make_float4(g.acc[mi][4][r], g.acc[mi][5][r], g.acc[mi][6][r], g.acc[mi][7][r]);
            float4* dst = reinterpret_cast<float4*>(y + size_t(t.row0 + row) * a.H + n0);
            dst[0] = lo;
            dst[1] = hi;
        }
}

template <int MI>
__global__ __launch_bounds__(256) void gemm2_kernel(FfnArgs a) {
    __shared__ __align__(16) uint16_t abuf[2 * StripGemm<MI>::kABufElems];
    // One-dimensional grid.  Workgroups go to the 8 XCDs round robin, so workgroup L runs on XCD L % 8; the
    // column workgroups of one (tile, K split) all read the same rows of h, so they are numbered to land on
    // one XCD back to back and find those rows in its L2 (on 8 XCDs each would fetch them from HBM again).
    const uint32_t n_cw = (a.H + 4 * kStrip - 1) / (4 * kStrip);
    const uint32_t xcd = blockIdx.x % 8u, q = blockIdx.x / 8u;
    const uint32_t col_wg = q % n_cw;
    const uint32_t pair = (q / n_cw) * 8u + xcd;             // (tile, split), tile-major
    if (pair >= a.tiles_cap * a.ksplit) return;
    const uint32_t tile = pair / a.ksplit, split = pair % a.ksplit;
    TileInfo t;
    if (!tile_info(a, tile, t)) return;
    if (MI > 1 && t.rows <= 16) gemm2_body<1>(a, t, abuf, col_wg, split);
    else if (MI > 2 && t.rows <= 32) gemm2_body<2>(a, t, abuf, col_wg, split);
    else if (MI > 4 && t.rows <= 64) gemm2_body<4>(a, t, abuf, col_wg, split);
    else if (MI > 6 && t.rows <= 96) gemm2_body<6>(a, t, abuf, col_wg, split);
    else gemm2_body<MI>(a, t, abuf, col_wg, split);
}

// ------------------------------------------------------------------ large row tiles (MFMA bound)
// When an expert sees hundreds of rows (prefill-shaped batches, the shared expert) the FFN is
// bound by the matrix cores, not by weight streaming, and operands must be reused from LDS.
// Workgroup tile 256 rows x 256 columns, k step 64, eight wavefronts as 4 (rows) x 2 (columns),
// two per SIMD so that one wavefront's LDS and barrier waits hide behind the other's MFMAs.
// Each wavefront owns 64 x 128 as 2 x 4 tiles of v_mfma_f32_32x32x16_bf16 (128 accumulator
// registers).  A rows (k contiguous) go to LDS as they are; B arrives row-major [k][n], so
// each lane transposes an 8 (k) x 4 (n) tile in registers (v_perm_b32) and writes [n][k] rows,
// after which both operands are read as 16-byte k-contiguous fragments.  LDS rows are padded
// by 16 bytes (conflict-free 16-byte reads); column c of a lane's tile goes to an LDS row
// chosen so that the 64 lanes of a write hit consecutive rows.  Two LDS buffers, one barrier
// per k step; the registers hold step s + 1 while step s is multiplied, are written to the
// other buffer between the MFMAs of step s and at once reloaded with step s + 2.
// Workgroups are numbered so that the 32 that run together on one XCD (one per CU) form a
// 4 x 8 block of tiles and share operand slices in that XCD's L2.
// MODE 1: the 256 tile columns are 128 of W1 and the same 128 of W3; a wavefront holds gate
// and up values of the same elements and applies SwiGLU in registers.  MODE 2: y = h W2.
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
constexpr int kTM = 256, kTK = 64, kLdsPitch = kTK + 8;   // pitch in BF16 elements
constexpr uint32_t kSuperM = 4, kSuperN = 8;              // tiles per super-tile (one XCD's 32 CUs)

template <int MODE>
__global__ __launch_bounds__(512) void gemm_tiled_kernel(FfnArgs a) {
    extern __shared__ __align__(16) uint16_t lds[];
    const uint32_t K = MODE == 1 ? a.H : a.F;
    const uint32_t N = MODE == 1 ? a.F : a.H;               // columns of one B matrix
    const uint32_t ncols_tile = MODE == 1 ? 128u : 256u;     // distinct output columns per tile
    const uint32_t n_ct = (N + ncols_tile - 1) / ncols_tile;
    const uint32_t n_rt = uint32_t(a.n_tiles[0]);
    const uint32_t n_sn = (n_ct + kSuperN - 1) / kSuperN;
    const uint32_t xcd = blockIdx.x % 8u, jj = blockIdx.x / 8u;
    const uint32_t st = (jj / (kSuperM * kSuperN)) * 8u + xcd;
    const uint32_t within = jj % (kSuperM * kSuperN);
    const uint32_t row_tile = (st / n_sn) * kSuperM + within / kSuperN;
    const uint32_t col_tile = (st % n_sn) * kSuperN + within % kSuperN;
    if (row_tile >= n_rt || col_tile >= n_ct) return;
    TileInfo t;
    if (!tile_info(a, row_tile, t)) return;
    const uint32_t n_base = col_tile * ncols_tile;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int q = lane & 31;
    constexpr int kTile = kTM * kLdsPitch;                   // LDS: [buffer][A tile | B tile]

    // global -> register staging.  A: 8 lanes cover one row's 64 k; rows tid / 8 + 64 i.
    const uint16_t* a_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int32_t r = min(int32_t(tid >> 3) + 64 * i, t.rows - 1);
        if (MODE == 1) {
            const int32_t pr = a.sorted_pair[t.row0 + r];
            a_src[i] = a.tokens + size_t(uint32_t(pr) / a.K) * a.H + 8 * (tid & 7);
        } else {
            a_src[i] = a.hbuf + size_t(t.row0 + r) * a.F + 8 * (tid & 7);
        }
    }
    const int a_dst = (tid >> 3) * kLdsPitch + 8 * (tid & 7);          // + 64 i rows
    // B: the lane's tile: 4 consecutive columns, 8 rows k = 8 (tid / 64) ..
    const uint32_t cg = tid & 63;
    const uint32_t bk = 8u * (tid >> 6);
    const uint16_t* b_src;
    int b_dst_row;                                           // + c * (MODE 1 ? 32 : 64) rows
    {
        const size_t mat = size_t(a.H) * a.F;
        if (MODE == 1) {
            const uint32_t col = min(n_base + 4u * (cg & 31u), N - 4);
            b_src = a.slots13 + size_t(t.slot) * 2 * mat + (cg >= 32 ? mat : 0) + col;
            b_dst_row = int(cg >> 5) * 128 + int(cg & 31);
        } else {
            const uint32_t col = min(n_base + 4u * cg, N - 4);
            b_src = a.slots2 + size_t(t.slot) * mat + col;
            b_dst_row = int(cg);
        }
    }
    constexpr int b_dst_step = MODE == 1 ? 32 : 64;
    const int b_dst = kTile + b_dst_row * kLdsPitch + int(bk);

    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // LDS fragment offsets of this wavefront (k-contiguous 16-byte reads).
    // MODE 2: B tile j = LDS rows 32 (4 wn + j) + q: column 4 (32 (j & 1) + q) + 2 wn + j / 2
    // MODE 1: j = 0, 1 gate, j = 2, 3 up: rows 128 (j / 2) + 32 (2 wn + j % 2) + q: column 4 q + 2 wn + j % 2
    const int kfrag = 8 * (lane >> 5);
    const int a_frag = (wm * 64 + q) * kLdsPitch + kfrag;                // + 32 i rows
    int b_frag[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = MODE == 1 ? ((j >> 1) * 128 + (2 * wn + (j & 1)) * 32 + q) : ((4 * wn + j) * 32 + q);
        b_frag[j] = kTile + row * kLdsPitch + kfrag;
    }

    u32x4 ga[4];
    u32x2 gb[8];
    const uint32_t n_steps = K / kTK;
    // item n of a step's 12 global loads: 0..3 the lane's A rows, 4..11 the 8 k rows of its B tile
    auto gload_item = [&](uint32_t k0, int n) __attribute__((always_inline)) {
        if (n < 4) ga[n] = *reinterpret_cast<const u32x4*>(a_src[n] + k0);
        else gb[n - 4] = *reinterpret_cast<const u32x2*>(b_src + size_t(k0 + bk + (n - 4)) * N);
    };
    // item n of a step's 8 LDS writes: 0..3 A rows, 4..7 column c = n - 4 of the transposed B tile
    auto lstore_item = [&](uint16_t* buf, int n) __attribute__((always_inline)) {
        if (n < 4) {
            *reinterpret_cast<u32x4*>(buf + a_dst + 64 * n * kLdsPitch) = ga[n];
        } else {
            const int c = n - 4;
            u32x4 v;
            const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
            v.x = __builtin_amdgcn_perm(gb[1][c >> 1], gb[0][c >> 1], sel);
            v.y = __builtin_amdgcn_perm(gb[3][c >> 1], gb[2][c >> 1], sel);
            v.z = __builtin_amdgcn_perm(gb[5][c >> 1], gb[4][c >> 1], sel);
            v.w = __builtin_amdgcn_perm(gb[7][c >> 1], gb[6][c >> 1], sel);
            *reinterpret_cast<u32x4*>(buf + b_dst + c * b_dst_step * kLdsPitch) = v;
        }
    };
    bf16x8 fa[2][2], fb[2][4];
    // item n of the 6 fragment reads of sub-step ks into register set `set`
    auto lfrag_item = [&](const uint16_t* buf, int ks, int set, int n) __attribute__((always_inline)) {
        if (n < 2) fa[set][n] = *reinterpret_cast<const bf16x8*>(buf + a_frag + 32 * n * kLdsPitch + ks * 16);
        else fb[set][n - 2] = *reinterpret_cast<const bf16x8*>(buf + b_frag[n - 2] + ks * 16);
    };
    auto mfma_item = [&](int set, int n) __attribute__((always_inline)) {
        const int i = n >> 2, j = n & 3;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    };

    // One k step.  STORE: refill the other buffer from the staging registers; LOAD: fetch step
    // s + 2 into them; NEXT: read the first fragments of the other buffer after the barrier.
    // A workgroup moves 64 KB per step through the vector memory path (64 B/clk per CU) and again
    // into LDS; issued in one burst, those instructions hold the issuing wavefronts for over a
    // thousand cycles while the matrix cores idle.  They are therefore issued one at a time
    // between the MFMAs (the scheduling barriers keep that order): the fragments of sub-step
    // ks + 1 and the 8 LDS writes during sub-step 0, the 12 global loads during sub-steps 1 and 2.
    // The step's barrier sits before the MFMAs of sub-step 3, which cover the first fragment
    // reads from the other buffer.
    auto step = [&](const uint16_t* cur, uint16_t* nxt, uint32_t k_next, auto STORE, auto LOAD, auto NEXT) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {                         // sub-step 0 (set 0)
            mfma_item(0, n);
            if (n < 6) lfrag_item(cur, 1, 1, n);
            if (STORE.value) lstore_item(nxt, n);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int n = 0; n < 8; ++n) {                         // sub-step 1 (set 1)
            mfma_item(1, n);
            if (n < 6) lfrag_item(cur, 2, 0, n);
            if (LOAD.value && n >= 2) gload_item(k_next, n - 2);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int n = 0; n < 8; ++n) {                         // sub-step 2 (set 0)
            mfma_item(0, n);
            if (n < 6) lfrag_item(cur, 3, 1, n);
            if (LOAD.value && n >= 2) gload_item(k_next, 6 + n - 2);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();                       // all reads of cur are in registers, nxt is complete
#pragma unroll
        for (int n = 0; n < 8; ++n) {                         // sub-step 3 (set 1)
            mfma_item(1, n);
            if (NEXT.value && n < 6) lfrag_item(nxt, 0, 0, n);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using Yes = std::integral_constant<bool, true>;
    using No = std::integral_constant<bool, false>;

#pragma unroll
    for (int n = 0; n < 12; ++n) gload_item(0, n);
#pragma unroll
    for (int n = 0; n < 8; ++n) lstore_item(lds, n);
    if (n_steps > 1) {
#pragma unroll
        for (int n = 0; n < 12; ++n) gload_item(kTK, n);
    }
    __syncthreads();
#pragma unroll
    for (int n = 0; n < 6; ++n) lfrag_item(lds, 0, 0, n);
    {
        uint16_t* cur = lds;
        uint16_t* nxt = lds + 2 * kTile;
        uint32_t s = 0;
        for (; s + 2 < n_steps; ++s) {
            step(cur, nxt, (s + 2) * kTK, Yes{}, Yes{}, Yes{});
            uint16_t* tmp = cur; cur = nxt; nxt = tmp;
        }
        if (s + 1 < n_steps) {
            step(cur, nxt, 0, Yes{}, No{}, Yes{});
            uint16_t* tmp = cur; cur = nxt; nxt = tmp;
        }
        step(cur, nxt, 0, No{}, No{}, No{});
    }

    // epilogue.  D layout of the 32x32 MFMA: column q = lane % 32, rows 8 (r / 4) + 4 (lane / 32) + r % 4
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int32_t row = wm * 64 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            if (row >= t.rows) continue;
            if (MODE == 1) {
                const uint32_t col = n_base + 4u * q + 2u * wn;      // two adjacent columns
                if (col >= N) continue;
                const uint32_t packed = pack_bf16_rne(swiglu(acc[i][0][r], acc[i][2][r]), swiglu(acc[i][1][r], acc[i][3][r]));
                *reinterpret_cast<uint32_t*>(a.hbuf + size_t(t.row0 + row) * a.F + col) = packed;
            } else {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const uint32_t col = n_base + 4u * (32 * half + q) + 2u * wn;
                    if (col >= N) continue;
                    *reinterpret_cast<float2*>(a.ybuf + size_t(t.row0 + row) * a.H + col) =
                        make_float2(acc[i][half][r], acc[i][half + 2][r]);
                }
            }
        }
}

// The same tiling with four wavefronts, one per SIMD, each owning 128 x 128 (4 x 4 MFMA tiles, 256
// accumulator registers).  LDS fragment traffic per flop falls by a third against the 64 x 128
// wavefront tile (a 128 x 128 tile reads 256 fragment rows per k for 16384 multiply-adds, the
// 64 x 128 one 192 for 8192), which is what bounds the eight-wavefront kernel.  With a single
// wavefront per SIMD nothing hides a wait, so the loop is software pipelined inside the
// wavefront: the fragments of sub-step ks + 1 are read while sub-step ks is multiplied, the
// refill of the other LDS buffer and the global loads of step s + 2 are spread over the MFMAs of
// sub-steps 0 and 1, and the step's only barrier sits before the MFMAs of sub-step 3, which then
// cover the first fragment reads from the other buffer.
template <int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_tiled4_kernel(FfnArgs a) {
    extern __shared__ __align__(16) uint16_t lds[];
    const uint32_t K = MODE == 1 ? a.H : a.F;
    const uint32_t N = MODE == 1 ? a.F : a.H;
    const uint32_t ncols_tile = MODE == 1 ? 128u : 256u;
    const uint32_t n_ct = (N + ncols_tile - 1) / ncols_tile;
    const uint32_t n_rt = uint32_t(a.n_tiles[0]);
    const uint32_t n_sn = (n_ct + kSuperN - 1) / kSuperN;
    const uint32_t xcd = blockIdx.x % 8u, jj = blockIdx.x / 8u;
    const uint32_t st = (jj / (kSuperM * kSuperN)) * 8u + xcd;
    const uint32_t within = jj % (kSuperM * kSuperN);
    const uint32_t row_tile = (st / n_sn) * kSuperM + within / kSuperN;
    const uint32_t col_tile = (st % n_sn) * kSuperN + within % kSuperN;
    if (row_tile >= n_rt || col_tile >= n_ct) return;
    TileInfo t;
    if (!tile_info(a, row_tile, t)) return;
    const uint32_t n_base = col_tile * ncols_tile;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int q = lane & 31;
    constexpr int kTile = kTM * kLdsPitch;

    // global -> register staging.  A: 8 lanes cover one row's 64 k; rows tid / 8 + 32 i.
    const uint16_t* a_base = MODE == 1 ? a.tokens : a.hbuf;
    uint32_t a_off[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int32_t r = min(int32_t(tid >> 3) + 32 * i, t.rows - 1);
        if (MODE == 1) {
            const int32_t pr = a.sorted_pair[t.row0 + r];
            a_off[i] = (uint32_t(pr) / a.K) * a.H + 8 * (tid & 7);
        } else {
            a_off[i] = uint32_t(t.row0 + r) * a.F + 8 * (tid & 7);
        }
    }
    const int a_dst = (tid >> 3) * kLdsPitch + 8 * (tid & 7);          // + 32 i rows
    // B: two lane tiles of 4 consecutive columns x 8 k rows: k = 8 (tid / 64) + 32 u
    const uint32_t cg = tid & 63;
    const uint32_t bk = 8u * (tid >> 6);
    const uint16_t* b_src;
    int b_dst_row;
    {
        const size_t mat = size_t(a.H) * a.F;
        if (MODE == 1) {
            const uint32_t col = min(n_base + 4u * (cg & 31u), N - 4);
            b_src = a.slots13 + size_t(t.slot) * 2 * mat + (cg >= 32 ? mat : 0) + col;
            b_dst_row = int(cg >> 5) * 128 + int(cg & 31);
        } else {
            const uint32_t col = min(n_base + 4u * cg, N - 4);
            b_src = a.slots2 + size_t(t.slot) * mat + col;
            b_dst_row = int(cg);
        }
    }
    constexpr int b_dst_step = MODE == 1 ? 32 : 64;
    const int b_dst = kTile + b_dst_row * kLdsPitch + int(bk);

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int kfrag = 8 * (lane >> 5);
    const int a_frag = (wm * 128 + q) * kLdsPitch + kfrag;              // + 32 i rows
    // B tile j of this wavefront: MODE 2 rows 32 (4 wn + j) + q; MODE 1 rows 128 (j / 2) + 32 (2 wn + j % 2) + q
    const int b_frag = kTile + (MODE == 1 ? (2 * wn * 32 + q) : (4 * wn * 32 + q)) * kLdsPitch + kfrag;
    auto b_frag_off = [](int j) { return (MODE == 1 ? ((j >> 1) * 128 + (j & 1) * 32) : (j * 32)) * kLdsPitch; };

    u32x4 ga[8];
    u32x2 gb[2][8];
    const uint32_t n_steps = K / kTK;
    // item n of a step's 24 global loads: 0..7 the lane's A rows, 8..23 the 2 x 8 k rows of its B tiles
    auto gload_item = [&](uint32_t k0, int n) __attribute__((always_inline)) {
        if (n < 8) ga[n] = *reinterpret_cast<const u32x4*>(a_base + a_off[n] + k0);
        else gb[(n - 8) >> 3][(n - 8) & 7] =
                 *reinterpret_cast<const u32x2*>(b_src + size_t(k0 + bk + 32 * ((n - 8) >> 3) + ((n - 8) & 7)) * N);
    };
    // item n of a step's 16 LDS writes: 0..7 A rows, 8..15 column c of transposed B tile u
    auto lstore_item = [&](uint16_t* buf, int n) __attribute__((always_inline)) {
        if (n < 8) {
            *reinterpret_cast<u32x4*>(buf + a_dst + 32 * n * kLdsPitch) = ga[n];
        } else {
            const int u = (n - 8) >> 2, c = (n - 8) & 3;
            u32x4 v;
            const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
            v.x = __builtin_amdgcn_perm(gb[u][1][c >> 1], gb[u][0][c >> 1], sel);
            v.y = __builtin_amdgcn_perm(gb[u][3][c >> 1], gb[u][2][c >> 1], sel);
            v.z = __builtin_amdgcn_perm(gb[u][5][c >> 1], gb[u][4][c >> 1], sel);
            v.w = __builtin_amdgcn_perm(gb[u][7][c >> 1], gb[u][6][c >> 1], sel);
            *reinterpret_cast<u32x4*>(buf + b_dst + 32 * u + c * b_dst_step * kLdsPitch) = v;
        }
    };
    bf16x8 fa[2][4], fb[2][4];
    // item n of the 8 fragment reads of sub-step ks into register set `set`
    auto lfrag_item = [&](const uint16_t* buf, int ks, int set, int n) __attribute__((always_inline)) {
        if (n < 4) fa[set][n] = *reinterpret_cast<const bf16x8*>(buf + a_frag + 32 * n * kLdsPitch + ks * 16);
        else fb[set][n - 4] = *reinterpret_cast<const bf16x8*>(buf + b_frag + b_frag_off(n - 4) + ks * 16);
    };
    auto mfma_item = [&](int set, int n) __attribute__((always_inline)) {
        const int i = n >> 2, j = n & 3;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    };

    // One k step.  STORE: refill the other buffer from the staging registers; LOAD: fetch step
    // s + 2 into them; NEXT: read the first fragments of the other buffer after the barrier.
    // Every memory instruction is issued between two MFMAs (the scheduling barriers keep that
    // order): the fragments of sub-step ks + 1 during sub-step ks, the 16 LDS writes during
    // sub-step 0, the 24 global loads during sub-steps 1 and 2.
    auto step = [&](const uint16_t* cur, uint16_t* nxt, uint32_t k_next, auto STORE, auto LOAD, auto NEXT) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < 16; ++n) {                        // sub-step 0 (set 0)
            mfma_item(0, n);
            if (n < 8) lfrag_item(cur, 1, 1, n);
            if (STORE.value) lstore_item(nxt, n);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int n = 0; n < 16; ++n) {                        // sub-step 1 (set 1)
            mfma_item(1, n);
            if (n < 8) lfrag_item(cur, 2, 0, n);
            if (LOAD.value && n >= 4) gload_item(k_next, n - 4);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int n = 0; n < 16; ++n) {                        // sub-step 2 (set 0)
            mfma_item(0, n);
            if (n < 8) lfrag_item(cur, 3, 1, n);
            if (LOAD.value && n >= 4) gload_item(k_next, 12 + n - 4);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();                       // all reads of cur are in registers, nxt is complete
#pragma unroll
        for (int n = 0; n < 16; ++n) {                        // sub-step 3 (set 1)
            mfma_item(1, n);
            if (NEXT.value && n < 8) lfrag_item(nxt, 0, 0, n);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using Yes = std::integral_constant<bool, true>;
    using No = std::integral_constant<bool, false>;

#pragma unroll
    for (int n = 0; n < 24; ++n) gload_item(0, n);
#pragma unroll
    for (int n = 0; n < 16; ++n) lstore_item(lds, n);
    if (n_steps > 1) {
#pragma unroll
        for (int n = 0; n < 24; ++n) gload_item(kTK, n);
    }
    __syncthreads();
#pragma unroll
    for (int n = 0; n < 8; ++n) lfrag_item(lds, 0, 0, n);
    uint16_t* cur = lds;
    uint16_t* nxt = lds + 2 * kTile;
    uint32_t s = 0;
    for (; s + 2 < n_steps; ++s) {
        step(cur, nxt, (s + 2) * kTK, Yes{}, Yes{}, Yes{});
        uint16_t* tmp = cur; cur = nxt; nxt = tmp;
    }
    if (s + 1 < n_steps) {
        step(cur, nxt, 0, Yes{}, No{}, Yes{});
        uint16_t* tmp = cur; cur = nxt; nxt = tmp;
    }
    step(cur, nxt, 0, No{}, No{}, No{});

#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int32_t row = wm * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            if (row >= t.rows) continue;
            if (MODE == 1) {
                const uint32_t col = n_base + 4u * q + 2u * wn;
                if (col >= N) continue;
                const uint32_t packed = pack_bf16_rne(swiglu(acc[i][0][r], acc[i][2][r]), swiglu(acc[i][1][r], acc[i][3][r]));
                *reinterpret_cast<uint32_t*>(a.hbuf + size_t(t.row0 + row) * a.F + col) = packed;
            } else {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const uint32_t col = n_base + 4u * (32 * half + q) + 2u * wn;
                    if (col >= N) continue;
                    *reinterpret_cast<float2*>(a.ybuf + size_t(t.row0 + row) * a.H + col) =
                        make_float2(acc[i][half][r], acc[i][half + 2][r]);
                }
            }
        }
}

// Third variant of the tiled kernel: both operands go from global memory straight into LDS
// (global_load_lds, 16 bytes per lane, no register staging, no LDS write instructions) and B stays
// row-major [k][n] there; its MFMA fragments are formed by the transposing LDS read
// (ds_read_b64_tr_b16: within 16 lanes, lane L receives element L % 4 of the four 8-byte groups that
// lanes L / 4, 4 + L / 4, 8 + L / 4, 12 + L / 4 point at).  Because an LDS-direct load fills 1 KiB
// contiguously (lane l at +16 l), rows cannot be padded; bank conflicts are avoided by choosing
// which global piece each lane fetches: A rows (128 bytes = 8 pieces) hold piece p ^ ((row >> 1) & 7)
// at position p; B rows (512 bytes = 8 units of 32 columns) hold unit u ^ (k & 3) at position u.
// LDS: [A stage 0 | A stage 1 | B stage 0 | B stage 1 | B stage 2], 32 KiB each = all 160 KiB.  Same
// eight wavefronts, wave tiles and sub-step schedule as gemm_tiled_kernel.
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
// Measurement aid, compile time only (python -m paper_2604_02715_amd.build -DFLUXMOE_D2L_PROBE=<bits>): parts of
// gemm_d2l_kernel's k loop left out to see what each costs.  The results are wrong with any bit set; every
// access that remains is one the full kernel makes too.  1: fragments are read from LDS once per tile only;
// 2: no A loads after the prologue; 4: no B loads after the prologue; 8: no waits for loads inside the loop
// (one wait after it); 16: every B load fetches the tile's first k block (stays cache resident).
#ifndef FLUXMOE_D2L_PROBE
#define FLUXMOE_D2L_PROBE 0
#endif

// WALK: a workgroup takes several tiles one after the other (see the tile loop at the end); without it the
// launch has one workgroup per tile number and the code for the upcoming tile falls away.
template <int MODE, int WAVES, bool WALK>
__global__ __launch_bounds__(WAVES * 64) void gemm_d2l_kernel(FfnArgs a) {
    // WAVES = 8: wavefronts 4 (rows) x 2 (columns), 64 x 128 each, two per SIMD.  WAVES = 4: 2 x 2,
    // 128 x 128 each (256 accumulator registers), one per SIMD: a third less LDS read traffic per MFMA.
    constexpr int kRowTiles = WAVES == 8 ? 2 : 4;            // 32-row MFMA tiles per wavefront
    constexpr int kWaveRows = 32 * kRowTiles;
    constexpr int kDma = 32 / WAVES;                         // 1 KiB loads per wavefront, operand and step
    constexpr int kMfma = 4 * kRowTiles;                     // MFMAs per sub-step
    constexpr int kFrag = kRowTiles + 8;                     // fragment reads per sub-step
    static_assert(WAVES == 8 || WAVES == 4, "wavefront layouts");
    extern __shared__ __align__(16) uint16_t lds[];
    const uint32_t K = MODE == 1 ? a.H : a.F;
    const uint32_t N = MODE == 1 ? a.F : a.H;
    const uint32_t ncols_tile = MODE == 1 ? 128u : 256u;
    const uint32_t n_ct = (N + ncols_tile - 1) / ncols_tile;
    const uint32_t n_rt = uint32_t(a.n_tiles[0]);
    // Super-tile of this launch: 32 tiles (one per CU of an XCD) as sm rows x sn columns, sn a power of two
    // chosen by the launcher so that the column tiles fill whole super-tiles where they can.
    const uint32_t sn_log2 = a.tiled_sn_log2, sn = 1u << sn_log2, sm = 32u >> sn_log2;
    const uint32_t n_sn = (n_ct + sn - 1) >> sn_log2;
    // Workgroups go to the 8 XCDs round robin, so (super-tile, K split) pair number p runs on XCD
    // p % 8: the splits of one super-tile land on different XCDs
    const uint32_t n_split = MODE == 2 ? a.ksplit : 1u;
    // Super-tiles are taken in groups of tiled_group super-rows (the row tiles of about one expert): for
    // each column block of the group, its super-rows run next to each other in time on different XCDs,
    // so the expert's weights for that column block leave HBM once and the other XCDs find them in the
    // memory-side cache, while the group's activations stay there across the column blocks.
    // (The second product has two column blocks at most and measured no gain: it keeps super-row order.)
    const uint32_t group = a.tiled_group;
    const uint32_t per_group = group * n_sn;
    // Tile number L -> (row tile, column tile, K split); false when the number names no tile.  A workgroup
    // takes the numbers blockIdx.x, blockIdx.x + gridDim.x, ...; gridDim.x is a multiple of 256 (or covers
    // all numbers), so all of them lie on the XCD that runs this workgroup and at the same place of
    // successive super-tiles.
    const uint32_t total = a.tiled_total;
    auto locate_unchecked = [&](uint32_t L, uint32_t& row_tile, uint32_t& col_tile, uint32_t& split) __attribute__((always_inline)) {
        const uint32_t xcd = L % 8u, jj = L / 8u;
        const uint32_t pair = (jj / 32u) * 8u + xcd;
        const uint32_t st = pair / n_split;
        split = pair % n_split;
        const uint32_t within = jj % 32u;
        const uint32_t grp = st / per_group, in_grp = st % per_group;
        row_tile = (grp * group + in_grp % group) * sm + (within >> sn_log2);
        col_tile = (in_grp / group) * sn + (within & (sn - 1u));
    };
    auto locate = [&](uint32_t L, uint32_t& row_tile, uint32_t& col_tile, uint32_t& split) __attribute__((always_inline)) {
        locate_unchecked(L, row_tile, col_tile, split);
        return row_tile < n_rt && col_tile < n_ct;
    };
    // A tile number together with what locate() says about it (the divisions in there are done on the
    // vector unit and take a third of a microsecond: once per tile is enough).
    struct TileId { uint32_t L, row_tile, col_tile, split; };
    // first number >= L of this workgroup's sequence that names a tile (L >= total when there is none)
    auto first_tile_from = [&](uint32_t L) __attribute__((always_inline)) {
        TileId id{L, 0, 0, 0};
        if (!WALK) {
            if (!(id.L < total && locate(id.L, id.row_tile, id.col_tile, id.split))) id.L = total;
            return id;
        }
        while (id.L < total && !locate(id.L, id.row_tile, id.col_tile, id.split)) id.L += gridDim.x;
        return id;
    };
    // its record (one 16-byte load; numbers past the end read record 0, which exists)
    auto load_rec = [&](const TileId& id) __attribute__((always_inline)) {
        return a.tile_rec[id.L < total ? id.row_tile : 0u];
    };

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    // The lane number as a value the compiler cannot trace back to threadIdx: what the per-tile set-up code
    // derives from it is then computed again for every tile instead of being held in registers across the
    // k loop, where registers are short.
    auto fresh_lane = [&]() __attribute__((always_inline)) {
        int x = tid;
        asm volatile("" : "+v"(x));
        return x & 63;
    };
    constexpr int kStageBytes = 32768;
    uint8_t* const lds_b8 = reinterpret_cast<uint8_t*>(lds);
    const size_t mat = size_t(a.H) * a.F;
    const uint32_t n_steps_all = K / kTK;

    // What a tile's loads need: the lane's byte offsets of its LDS-direct loads (kDma for A, kDma for B
    // per step) from bases that are uniform over the workgroup, the step range, where the results go.
    struct TileState {
        uint32_t a_off[kDma], b_off[kDma];   // until finish_state(): a_off = pair numbers of the lane's rows as loaded
                                             // (first product) or their row numbers (second), b_off unset
        const uint8_t* a_base;
        const uint8_t* b_base;
        int32_t rows, row0;
        uint32_t n_base, split, n_steps;
        bool valid;
    };
    // rec: the tile's record, loaded earlier.  Issues the gather of the rows' pair numbers (first product);
    // finish_state() turns them into offsets where the tile's first loads are issued, so that nothing waits
    // for the gather in between.
    auto make_state = [&](const TileId& id, const int4& rec, TileState& s) __attribute__((always_inline)) {
        const uint32_t col_tile = id.col_tile, split = id.split;
        s.valid = id.L < total;
        s.rows = __builtin_amdgcn_readfirstlane(rec.z);
        s.row0 = __builtin_amdgcn_readfirstlane(rec.y);
        const int32_t slot = __builtin_amdgcn_readfirstlane(rec.w);
        s.valid = s.valid && s.rows > 0 && slot >= 0;
        if (!s.valid) { s.rows = 1; s.row0 = 0; }
        s.n_base = col_tile * ncols_tile;
        s.split = split;
        // split K (second product only): this tile multiplies steps [step_lo, step_hi) of the K / 64
        // and writes its own FP32 partial, which combine_kernel sums in split order
        const uint32_t step_lo = uint32_t(uint64_t(n_steps_all) * split / n_split);
        const uint32_t step_hi = uint32_t(uint64_t(n_steps_all) * (split + 1) / n_split);
        const uint32_t k_begin = step_lo * kTK;
        s.n_steps = MODE == 1 ? 0u : step_hi - step_lo;        // >= 1: the host keeps ksplit <= K / 64
        s.a_base = MODE == 1 ? nullptr : reinterpret_cast<const uint8_t*>(a.hbuf) + size_t(k_begin) * 2;
        const int lane = fresh_lane();
#pragma unroll
        for (int i = 0; i < kDma; ++i) {
            const int r_lds = 8 * (wave * kDma + i) + (lane >> 3);                 // row of the A tile
            const int32_t r = min(r_lds, s.rows - 1);
            s.a_off[i] = MODE == 1 ? uint32_t(a.sorted_pair[s.row0 + r]) : uint32_t(s.row0 + r);
        }
        const size_t slot_u = s.valid ? size_t(slot) : 0u;
        s.b_base = reinterpret_cast<const uint8_t*>(
            MODE == 1 ? a.slots13 + slot_u * 2 * mat : a.slots2 + slot_u * mat + size_t(k_begin) * N);
    };
    auto finish_state = [&](TileState& s) __attribute__((always_inline)) {
        const int lane = fresh_lane();
#pragma unroll
        for (int i = 0; i < kDma; ++i) {
            const int r_lds = 8 * (wave * kDma + i) + (lane >> 3);              // row of the A tile
            const int piece = (lane & 7) ^ ((r_lds >> 1) & 7);                  // global 16-byte piece held at position lane & 7
            const uint32_t row_elems = MODE == 1 ? (s.a_off[i] / a.K) * a.H : s.a_off[i] * a.F;
            s.a_off[i] = 2u * (row_elems + 8u * piece);
        }
#pragma unroll
        for (int i = 0; i < kDma; ++i) {
            const int k_lds = 2 * (wave * kDma + i) + (lane >> 5);                 // k row of the B tile
            const int pp = lane & 31;                                           // physical 16-byte piece in the row
            const int unit = (pp >> 2) ^ (k_lds & 3);                           // logical unit of 32 columns
            const uint32_t c = 32u * unit + 8u * (pp & 3);                      // column inside the 256-column tile
            uint32_t elems;
            if (MODE == 1) elems = (c >= 128 ? uint32_t(mat) : 0u) + min(s.n_base + (c & 127u), N - 8);
            else elems = min(s.n_base + c, N - 8);
            s.b_off[i] = 2u * (elems + uint32_t(k_lds) * N);
        }
    };
    // stage_off: 0 or kStageBytes, uniform.  The load is written as inline assembly on purpose: with
    // the compiler's builtin, every later LDS read waits for all outstanding LDS-direct loads
    // (it cannot see that they go to the other stage), which serialises the whole step.  Here the
    // only waits are the explicit ones before the barriers.
    const uint32_t lds_base = uint32_t(uintptr_t((__attribute__((address_space(3))) void*)lds));
    // (M0 carries the LDS destination and is read when the instruction issues; it is a register the
    // compiler reserves, so its previous value is put back.)
    auto dma16 = [&](const uint8_t* gptr, uint32_t lds_addr) __attribute__((always_inline)) {
        uint32_t saved_m0;
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                     : "=&s"(saved_m0) : "v"(gptr), "s"(lds_addr) : "memory");
    };
    // a_stage_off / b_stage_off: byte offset of the destination stage inside the operand's region, uniform
    auto dma_a = [&](const TileState& s, uint32_t k0, int a_stage_off, int n) __attribute__((always_inline)) {
        // (the first product never splits K: its A base and step count are the same for every tile)
        const uint8_t* base = MODE == 1 ? reinterpret_cast<const uint8_t*>(a.tokens) : s.a_base;
        dma16(base + size_t(k0) * 2 + s.a_off[n], lds_base + a_stage_off + (wave * kDma + n) * 1024);
    };
    auto dma_b = [&](const TileState& s, uint32_t k0, int b_stage_off, int n) __attribute__((always_inline)) {
        dma16(s.b_base + size_t((FLUXMOE_D2L_PROBE & 16) ? 0u : k0) * N * 2 + s.b_off[n], lds_base + 2 * kStageBytes + b_stage_off + (wave * kDma + n) * 1024);
    };
    auto steps_of = [&](const TileState& s) __attribute__((always_inline)) { return MODE == 1 ? n_steps_all : s.n_steps; };
    // a tile's first loads: A and B of steps 0 and 1 into stages 0 and 1 (B of step 2 is issued by step 0)
    auto prime = [&](const TileState& s) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < kDma; ++n) { dma_a(s, 0, 0, n); dma_b(s, 0, 0, n); }
        if (steps_of(s) > 1) {
#pragma unroll
            for (int n = 0; n < kDma; ++n) { dma_a(s, kTK, kStageBytes, n); dma_b(s, kTK, kStageBytes, n); }
        }
    };

    // ---- fragment addresses (bytes from the start of stage 0 of the operand's region); the k loop moves
    // them from stage to stage, so every tile starts from these values again
    int a_addr[kRowTiles][4];
    int b_addr[4];
    f32x16 acc[kRowTiles][4];
    int b_next_delta = kStageBytes;
    int a_own = 0, b_own = 0;                                // byte offsets of the current step's stages
    auto begin_tile = [&]() __attribute__((always_inline)) {
        const int lane = fresh_lane();
        const int q = lane & 31, h = lane >> 5;
        const int e = (lane & 15) >> 2, g = lane & 3, nh = (lane >> 4) & 1;
#pragma unroll
        for (int i = 0; i < kRowTiles; ++i) {
            const int R = wm * kWaveRows + 32 * i + q;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) a_addr[i][ks] = R * 128 + 16 * ((2 * ks + h) ^ ((R >> 1) & 7));
        }
        // B fragment j of sub-step ks, read t: row 16 ks + 8 h + 4 t + e, unit u(j) ^ e, bytes 32 nh + 8 g
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int unit = MODE == 1 ? ((((2 * wn + (j & 1)) ^ e)) + 4 * (j >> 1)) : (4 * wn + (j ^ e));
            b_addr[j] = 2 * kStageBytes + (8 * h + e) * 512 + 64 * unit + 32 * nh + 8 * g;
        }
#pragma unroll
        for (int i = 0; i < kRowTiles; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        b_next_delta = kStageBytes;
        a_own = 0;
        b_own = 0;
    };

    bf16x8 fa[2][kRowTiles];
    i16x4 fb_lo[2][4], fb_hi[2][4];
    // item n of the kFrag fragment reads of sub-step ks from `stage` into register set `set`: first the
    // A tiles, then the two halves (k 0..3 and 4..7 of the lane's 8) of the four B fragments
    // OTHER: read from the next step's stage instead of the one the address registers point at
    // (A: the other of two stages; B: b_next_delta bytes further in its ring of three)
    auto lfrag_item = [&](int other, int ks, int set, int n) __attribute__((always_inline)) {
        if (n < kRowTiles) {
            fa[set][n] = *reinterpret_cast<const bf16x8*>(lds_b8 + (a_addr[n][ks] ^ (other ? kStageBytes : 0)));
        } else {
            const int j = (n - kRowTiles) >> 1, tt = (n - kRowTiles) & 1;
            const i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (lds_i16x4*)(lds_b8 + ((b_addr[j] + (other ? b_next_delta : 0)) + ks * 8192 + tt * 2048)));
            if (tt == 0) fb_lo[set][j] = v; else fb_hi[set][j] = v;
        }
    };
    typedef short i16x8 __attribute__((ext_vector_type(8)));
    auto mfma_item = [&](int set, int n) __attribute__((always_inline)) {
        const int i = n >> 2, j = n & 3;
        const i16x8 full = __builtin_shufflevector(fb_lo[set][j], fb_hi[set][j], 0, 1, 2, 3, 4, 5, 6, 7);
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], __builtin_bit_cast(bf16x8, full), acc[i][j], 0, 0, 0);
    };

    // Step s multiplies A stage s % 2 and B stage s % 3.  After its barrier nobody reads those
    // stages any more, so sub-step 3 issues the A loads of step s + 2 into the same A stage and
    // sub-step 0 of the next step issues the B loads of step s + 3 into the same B stage: B, whose
    // first reader in an XCD goes to HBM, is fetched two steps ahead, A (mostly L2 hits) one.
    // Loads return in order, so waiting until at most 4 are outstanding before the barrier of
    // step s leaves only the B loads of step s + 2 in flight.
    // LOAD_B: B of step s + 2 (issued in sub-step 0); LOAD_A: A of step s + 2 (after the barrier);
    // NEXT: another step follows.  After the barrier of a tile's last step all five stages are free: that
    // step issues the first loads of the workgroup's next tile (`upcoming`, if it has one) behind its last
    // MFMAs, and they travel while the epilogue runs.
    auto step = [&](const TileState& cur, TileState& upcoming, uint32_t k0, auto LOAD_B, auto LOAD_A, auto NEXT, auto ACT) __attribute__((always_inline)) {
        const int b_plus2 = b_own >= kStageBytes ? b_own - kStageBytes : b_own + 2 * kStageBytes;   // stage of step s + 2
        // one sub-step: the MFMAs of register set `set`, between them the fragment reads of sub-step
        // next_ks into the other set (other = 1: from the next step's stages) and this step's share of loads
        auto sub = [&](int set, int other, int next_ks, auto READ, auto DMA_B, auto DMA_A) __attribute__((always_inline)) {
#pragma unroll
            for (int n = 0; n < kMfma; ++n) {
                if (ACT.value) mfma_item(set, n);
                if (READ.value && ACT.value && n < kFrag && !(FLUXMOE_D2L_PROBE & 1)) lfrag_item(other, next_ks, set ^ 1, n);
                if (DMA_B.value && (n & 1) && !(FLUXMOE_D2L_PROBE & 4)) dma_b(cur, k0 + 2 * kTK, b_plus2, n >> 1);
                if (DMA_A.value && (n & 1) && !(FLUXMOE_D2L_PROBE & 2)) dma_a(cur, k0 + 2 * kTK, a_own, n >> 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (READ.value && ACT.value && !(FLUXMOE_D2L_PROBE & 1)) {
#pragma unroll
                for (int n = kMfma; n < kFrag; ++n) lfrag_item(other, next_ks, set ^ 1, n);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        using T = std::integral_constant<bool, true>;
        using F = std::integral_constant<bool, false>;
        sub(0, 0, 1, T{}, LOAD_B, F{});                       // sub-step 0
        sub(1, 0, 2, T{}, F{}, F{});                          // sub-step 1
        sub(0, 0, 3, T{}, F{}, F{});                          // sub-step 2
        if (!(FLUXMOE_D2L_PROBE & 8)) {
            if (LOAD_B.value) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kDma) : "memory");   // all but this step's own B loads have landed
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __syncthreads();                                      // all reads of this step's stages are in registers
        sub(1, 1, 0, NEXT, F{}, LOAD_A);                      // sub-step 3
        if (WALK && !NEXT.value && upcoming.valid) { finish_state(upcoming); prime(upcoming); }
        // advance to the next step's stages
#pragma unroll
        for (int i = 0; i < kRowTiles; ++i)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) a_addr[i][ks] ^= kStageBytes;
#pragma unroll
        for (int j = 0; j < 4; ++j) b_addr[j] += b_next_delta;
        a_own ^= kStageBytes;
        b_own = b_own == 2 * kStageBytes ? 0 : b_own + kStageBytes;
        b_next_delta = b_own == 2 * kStageBytes ? -2 * kStageBytes : kStageBytes;
    };
    using Yes = std::integral_constant<bool, true>;
    using No = std::integral_constant<bool, false>;

    auto epilogue = [&](const TileState& c) __attribute__((always_inline)) {
    const int lane = fresh_lane();
    const int q = lane & 31, h = lane >> 5;
    // epilogue.  D layout of the 32x32 MFMA: column q = lane % 32, rows 8 (r / 4) + 4 (lane / 32) + r % 4;
    // fragment j of this wavefront holds tile columns 128 wn + 32 j + q (MODE 2) or, in MODE 1,
    // gate (j = 0, 1) and up (j = 2, 3) of h columns 64 wn + 32 (j & 1) + q
    if (MODE == 1) {
        // a lane holds one h column; neighbouring lanes swap values (DPP) so that even lanes store
        // columns (q, q + 1) of an even row and odd lanes columns (q - 1, q) of the next row: 4-byte
        // stores instead of 2-byte ones
        // v_perm_b32(other, own, sel): selector bytes 0..3 pick from own, 4..7 from other
        const uint32_t pair_sel = (q & 1) ? 0x03020706u : 0x05040100u;
        // one 64-bit address per stored row; the two column groups of a row lie 64 bytes apart
        const uint32_t col0 = c.n_base + 64u * wn + (q & ~1);
        uint16_t* const hlane = a.hbuf + size_t(c.row0) * a.F + col0;
#pragma unroll
        for (int i = 0; i < kRowTiles; ++i)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const int32_t row = wm * kWaveRows + i * 32 + (r >> 2) * 8 + h * 4 + (r & 3) + (q & 1);
                uint16_t* const hrow = hlane + size_t(uint32_t(row)) * a.F;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    // own = (row r, row r + 1) of this lane's column; the neighbouring lane's pair comes by DPP
                    // (quad_perm 1,0,3,2); an even lane keeps both lanes' row-r values, an odd lane both
                    // lanes' row-(r + 1) values, lower column first: one byte permute with a per-lane selector
                    const uint32_t own = pack_bf16_rne(swiglu(acc[i][j][r], acc[i][j + 2][r]),
                                                       swiglu(acc[i][j][r + 1], acc[i][j + 2][r + 1]));
                    const uint32_t other = uint32_t(__builtin_amdgcn_update_dpp(0, int(own), 0xB1, 0xF, 0xF, true));
                    const uint32_t packed = __builtin_amdgcn_perm(other, own, pair_sel);
                    if (row < c.rows && col0 + 32u * j < N)
                        *reinterpret_cast<uint32_t*>(hrow + 32 * j) = packed;
                }
            }
    } else {
        // one 64-bit address per stored row; the four column groups of a row lie 128 bytes apart
        const uint32_t col0 = c.n_base + 128u * wn + q;
        float* const ylane = a.ybuf + (size_t(c.split) * a.pairs_cap + size_t(c.row0)) * a.H + col0;
#pragma unroll
        for (int i = 0; i < kRowTiles; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int32_t row = wm * kWaveRows + i * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
                if (row >= c.rows) continue;
                float* const yrow = ylane + size_t(uint32_t(row)) * a.H;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (col0 + 32u * j >= N) continue;
                    yrow[32 * j] = acc[i][j][r];
                }
            }
    }
    };

    // A wavefront whose 64 rows all lie past the tile's last row (tail tiles of an expert) takes part
    // in the loads and barriers only: with at most 128 rows every SIMD runs one multiplying wavefront
    // instead of two.
    auto k_loop = [&](const TileState& cur, TileState& upcoming, auto ACT) __attribute__((always_inline)) {
        if (ACT.value) {
#pragma unroll
            for (int n = 0; n < kFrag; ++n) lfrag_item(0, 0, 0, n);
            if (FLUXMOE_D2L_PROBE & 1) {
#pragma unroll
                for (int n = 0; n < kFrag; ++n) lfrag_item(0, 1, 1, n);
            }
        }
        uint32_t s = 0;
        const uint32_t n_steps = steps_of(cur);
        for (; s + 2 < n_steps; ++s) step(cur, upcoming, s * kTK, Yes{}, Yes{}, Yes{}, ACT);
        if (s + 1 < n_steps) step(cur, upcoming, s * kTK, No{}, No{}, Yes{}, ACT);
        step(cur, upcoming, 0, No{}, No{}, No{}, ACT);
    };

    // ---- the workgroup's tiles.  Three of them are in the pipeline: `cur` is multiplied; `nxt` has had its
    // record read and its row gather issued (the values are first touched when its loads are issued at the
    // end of cur's k loop); the record of the one after is on its way.
    // (the record of the workgroup's own number is requested before anything looks at the tile count, which
    // is itself a load: the two travel together instead of one after the other)
    int4 rec_own;
    {
        TileId own{blockIdx.x, 0, 0, 0};
        uint32_t c, sp;
        locate_unchecked(own.L, own.row_tile, c, sp);
        rec_own = a.tile_rec[min(own.row_tile, a.tiles_cap - 1u)];
    }
    const TileId none{total, 0, 0, 0};
    TileId id_cur = first_tile_from(blockIdx.x);
    TileId id_nxt = WALK ? first_tile_from(id_cur.L < total ? id_cur.L + gridDim.x : total) : none;
    int4 rec_nxt = WALK ? load_rec(id_nxt) : make_int4(0, 0, 0, -1);
    TileState cur, nxt;
    make_state(id_cur, id_cur.L == blockIdx.x ? rec_own : load_rec(id_cur), cur);
    nxt.valid = false;
    bool primed = false;                                     // cur's first loads were issued by the tile before it
    while (id_cur.L < total) {
        TileId id_after = none;
        int4 rec_after = make_int4(0, 0, 0, -1);
        if (WALK) {
            id_after = first_tile_from(id_nxt.L < total ? id_nxt.L + gridDim.x : total);
            rec_after = load_rec(id_after);                 // the one load between cur's first loads and the wait below
        }
        // The upcoming tile's row gather is issued here, a whole k loop before its values are needed: issued
        // later (between the steady steps and the last two) the in-order wait of the next step stalls on it
        // (measured: 10 % of the first product's time).
        if (WALK) make_state(id_nxt, rec_nxt, nxt);
        if (cur.valid) {
            begin_tile();
            if (!primed) {
                finish_state(cur);
                prime(cur);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            } else {
                // loads return in order: cur's first loads are older than the record load and the gather just issued
                asm volatile("s_waitcnt vmcnt(%0)" :: "n"(MODE == 1 ? 1 + kDma : 1) : "memory");
            }
            __syncthreads();
            if (wm * kWaveRows < cur.rows) k_loop(cur, nxt, Yes{}); else k_loop(cur, nxt, No{});
            if (FLUXMOE_D2L_PROBE & 8) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); __syncthreads(); }
            epilogue(cur);
        }
        if (!WALK) break;
        primed = cur.valid && nxt.valid;
        cur = nxt;
        id_cur = id_nxt;
        id_nxt = id_after;
        rec_nxt = rec_after;
    }
}

// out[t][:] (+)= sum_k gate * sum_split y
template <uint32_t kGroup>
__global__ __launch_bounds__(256) void combine_kernel(FfnArgs a) {
    const uint32_t tok = blockIdx.y;
    const uint32_t h = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (h >= a.H) return;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    float* o = a.out + size_t(tok) * a.H + h;
    if (a.flags & 1u) s = *reinterpret_cast<const float4*>(o);
    // kGroup pairs of the token at a time (the launcher takes the smallest of 2, 4, 8, 16 that covers top-k,
    // 16 beyond): their positions and gates are fetched together, then their rows of y, so that the loads
    // overlap instead of following each other pair by pair.  A skipped pair, and a place of the group past
    // top-k, reads row 0 (a cache hit) and adds nothing; the sums run over the splits and then over k, in that
    // order, whatever the group size.
    for (uint32_t k0 = 0; k0 < a.K; k0 += kGroup) {
        int32_t pos[kGroup];
        float gate[kGroup];
#pragma unroll
        for (uint32_t j = 0; j < kGroup; ++j) {
            const bool in = k0 + j < a.K;
            pos[j] = in ? a.pair_pos[tok * a.K + k0 + j] : -1;
            gate[j] = in ? a.topk_w[tok * a.K + k0 + j] : 0.f;
        }
        float4 y[kGroup];
#pragma unroll
        for (uint32_t j = 0; j < kGroup; ++j) y[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (uint32_t sp = 0; sp < a.ksplit; ++sp) {
            float4 v[kGroup];
#pragma unroll
            for (uint32_t j = 0; j < kGroup; ++j)
                v[j] = *reinterpret_cast<const float4*>(a.ybuf + (size_t(sp) * a.pairs_cap + uint32_t(max(pos[j], 0))) * a.H + h);
#pragma unroll
            for (uint32_t j = 0; j < kGroup; ++j) {
                if (pos[j] >= 0) { y[j].x += v[j].x; y[j].y += v[j].y; y[j].z += v[j].z; y[j].w += v[j].w; }
            }
        }
#pragma unroll
        for (uint32_t j = 0; j < kGroup; ++j) {
            if (pos[j] >= 0) { s.x += gate[j] * y[j].x; s.y += gate[j] * y[j].y; s.z += gate[j] * y[j].z; s.w += gate[j] * y[j].w; }
        }
    }
    *reinterpret_cast<float4*>(o) = s;
}

// Measurement aid: nothing but independent 32x32x16 BF16 MFMAs (16 accumulators per wavefront, one
// wavefront per SIMD) on operands read once from `in`: what the matrix cores sustain on this chip
// for a given operand content, with no memory traffic in the loop.
__global__ __launch_bounds__(256) void mfma_probe_kernel(const u32x4* in, float* out, uint32_t iters) {
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    union { u32x4 u; bf16x8 v; } fa[4], fb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        fa[i].u = in[(threadIdx.x * 8 + i) & 4095];
        fb[i].u = in[(threadIdx.x * 8 + 4 + i + blockIdx.x) & 4095];
    }
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[j].v, acc[i * 4 + j], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = sum;
}

}  // namespace

hipError_t launch_mfma_probe(const void* operands, float* out, uint32_t n_workgroups, uint32_t iters,
                             hipStream_t stream) {
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(n_workgroups), dim3(256), 0, stream,
                       static_cast<const u32x4*>(operands), out, iters);
    return hipGetLastError();
}

hipError_t launch_ffn(const FfnArgs& args, int n_cus, hipStream_t stream, SpanHook hook, void* user) {
    (void)n_cus;
    if (args.T == 0) return hipSuccess;
    FfnArgs a = args;
    auto mark = [&](int kind, int begin) { if (hook) hook(user, kind, begin, stream); };
    const size_t sh = (3 * size_t(a.E) + 1024) * sizeof(int32_t);
    mark(1, 1);
    if (a.n_chunks) {
        hipLaunchKernelGGL(route_count_kernel, dim3(a.n_chunks), dim3(1024), size_t(a.E) * sizeof(int32_t), stream, a);
        hipLaunchKernelGGL(route_sort_kernel<true>, dim3(1), dim3(1024), sh, stream, a);
        hipLaunchKernelGGL(route_scatter_kernel, dim3(a.n_chunks), dim3(1024), size_t(a.E) * sizeof(int32_t), stream, a);
    } else {
        hipLaunchKernelGGL(route_sort_kernel<false>, dim3(1), dim3(1024), sh, stream, a);
    }
    mark(1, 0);
    auto launch_combine = [&](dim3 grid) {
        if (a.K <= 2) hipLaunchKernelGGL(combine_kernel<2>, grid, dim3(256), 0, stream, a);
        else if (a.K <= 4) hipLaunchKernelGGL(combine_kernel<4>, grid, dim3(256), 0, stream, a);
        else if (a.K <= 8) hipLaunchKernelGGL(combine_kernel<8>, grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL(combine_kernel<16>, grid, dim3(256), 0, stream, a);
    };
    const uint32_t strips1 = (a.F + kStrip - 1) / kStrip;
    const uint32_t strips2 = (a.H + kStrip - 1) / kStrip;
    const dim3 g1((strips1 + 1) / 2, a.tiles_cap, 1);
    const dim3 g2(((a.tiles_cap * a.ksplit + 7) / 8 * 8) * ((strips2 + 3) / 4), 1, 1);
    if (a.m_tile == 256) {
        const size_t lds_bytes = 4 * size_t(kTM) * kLdsPitch * sizeof(uint16_t);
        const bool four = a.tiled_waves == 4;
        const bool d2l4 = a.tiled_waves == 1;                       // LDS-direct loads, four wavefronts of 128 x 128
        const bool d2l = a.tiled_waves == 2 || d2l4;
        if (!d2l && a.ksplit != 1) return hipErrorInvalidValue;     // only the LDS-direct kernels split K
        if (a.ksplit == 0 || a.ksplit > a.F / kTK) return hipErrorInvalidValue;
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_tiled_kernel<1>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, int(lds_bytes));
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_tiled_kernel<2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, int(lds_bytes));
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_tiled4_kernel<1>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, int(lds_bytes));
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_tiled4_kernel<2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, int(lds_bytes));
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_d2l_kernel<1, 8, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 163840);
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_d2l_kernel<2, 8, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 163840);
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_d2l_kernel<1, 4, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 163840);
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_d2l_kernel<2, 4, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 163840);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        mark(2, 1);
        // register-staged kernels: super-tiles of 4 x 8 tiles, super-row order
        auto grid_for = [&](uint32_t n_ct) {
            const uint32_t n_sm = (a.tiles_cap + kSuperM - 1) / kSuperM;
            const uint32_t n_sn = (n_ct + kSuperN - 1) / kSuperN;
            const uint32_t supers = (n_sm * n_sn + 7) / 8 * 8;                // whole rounds over the 8 XCDs
            return dim3(supers * kSuperM * kSuperN, 1, 1);
        };
        // LDS-direct kernels.  A launch whose workgroups walk through the tiles takes as the super-tile's
        // column count the power of two (8, 4, 16, 2 in that order of preference) that leaves the fewest empty
        // places in the last column block: a workgroup whose place is empty there has nothing to do while the
        // others work (H 5120 / F 1536, 12 column tiles of the first product: 4 x 8 super-tiles 10.2 ms,
        // 8 x 4 8.1 ms at 2048 rows per expert).  With one workgroup per tile the dispatcher fills the holes
        // and 4 x 8 measured best.  A group is about one expert's super-rows (first product only; at most 8,
        // one per XCD).  Sets the launch's fields in `a`.
        const uint64_t pairs_all = uint64_t(a.T) * a.K;
        const uint64_t avg_rows = pairs_all / std::max<uint64_t>(1, std::min<uint64_t>(a.E, pairs_all));
        auto d2l_all = [&](uint32_t n_ct, uint32_t n_split, bool grouped, bool walk) {
            uint32_t best_log2 = 3, best_pad = ~0u;
            for (uint32_t lg : {3u, 2u, 4u, 1u}) {
                if (!walk && lg != 3u) continue;
                const uint32_t pad = ((n_ct + (1u << lg) - 1) >> lg << lg) - n_ct;
                if (pad < best_pad) { best_pad = pad; best_log2 = lg; }
            }
            a.tiled_sn_log2 = best_log2;
            const uint32_t sm = 32u >> best_log2;
            const uint64_t per_super_row = 256ull * sm;
            a.tiled_group = !grouped ? 1u : uint32_t(std::min<uint64_t>(8, std::max<uint64_t>(1,
                args.tiled_group ? args.tiled_group : (avg_rows + per_super_row / 2) / per_super_row)));
            const uint32_t n_sm = ((a.tiles_cap + sm - 1) / sm + a.tiled_group - 1) / a.tiled_group * a.tiled_group;
            const uint32_t n_sn = (n_ct + (1u << best_log2) - 1) >> best_log2;
            const uint32_t supers = (n_sm * n_sn * n_split + 7) / 8 * 8;      // whole rounds over the 8 XCDs
            return dim3(supers * 32u, 1, 1);
        };
        // LDS-direct kernels: the launch covers `tiled_total` tile numbers; a workgroup walks through the numbers
        // blockIdx.x, + gridDim.x, ... and overlaps a tile's epilogue with the next one's first loads.  One
        // workgroup fits on a CU, so the first product runs tiled_persist x 256 workgroups (a multiple of 256
        // keeps a workgroup's numbers on its XCD); with tiled_persist = 0, and for the second product, one
        // workgroup per number.  The fixed hand-out loses when the last column block of a super-tile row is
        // partly empty (workgroups with no tile there idle): measured on H 5120 / F 1536, 2048 rows per expert,
        // the first product gains 7 % (its tiles are short: 80 steps, and each needs a row gather first), the
        // second, whose 20 column tiles leave half of every third block empty, loses 11 %; on H 4096 / F 14336
        // both change by under 1 %.
        auto d2l_grid = [&](const dim3& all, bool walk) {
            a.tiled_total = all.x;
            const uint32_t cap = a.tiled_persist * 256u;
            return (walk && a.tiled_persist && all.x > cap) ? dim3(cap, 1, 1) : all;
        };
        if (d2l4) { const dim3 g = d2l_grid(d2l_all((a.F + 127) / 128, 1, true, false), false); hipLaunchKernelGGL((gemm_d2l_kernel<1, 4, false>), g, dim3(256), 163840, stream, a); }
        else if (d2l) { const dim3 g = d2l_grid(d2l_all((a.F + 127) / 128, 1, true, a.tiled_persist != 0), true); hipLaunchKernelGGL((gemm_d2l_kernel<1, 8, true>), g, dim3(512), 163840, stream, a); }
        else if (four) hipLaunchKernelGGL(gemm_tiled4_kernel<1>, grid_for((a.F + 127) / 128), dim3(256), lds_bytes, stream, a);
        else hipLaunchKernelGGL(gemm_tiled_kernel<1>, grid_for((a.F + 127) / 128), dim3(512), lds_bytes, stream, a);
        mark(2, 0);
        mark(3, 1);
        if (d2l4) { const dim3 g = d2l_grid(d2l_all((a.H + 255) / 256, a.ksplit, false, false), false); hipLaunchKernelGGL((gemm_d2l_kernel<2, 4, false>), g, dim3(256), 163840, stream, a); }
        else if (d2l) { const dim3 g = d2l_grid(d2l_all((a.H + 255) / 256, a.ksplit, false, false), false); hipLaunchKernelGGL((gemm_d2l_kernel<2, 8, false>), g, dim3(512), 163840, stream, a); }
        else if (four) hipLaunchKernelGGL(gemm_tiled4_kernel<2>, grid_for((a.H + 255) / 256), dim3(256), lds_bytes, stream, a);
        else hipLaunchKernelGGL(gemm_tiled_kernel<2>, grid_for((a.H + 255) / 256), dim3(512), lds_bytes, stream, a);
        mark(3, 0);
        const dim3 gc2((a.H / 4 + 255) / 256, a.T, 1);
        mark(4, 1);
        launch_combine(gc2);
        mark(4, 0);
        return hipGetLastError();
    }
    if (a.m_tile != 16 && a.m_tile != 32 && a.m_tile != 64 && a.m_tile != 96 && a.m_tile != 128) return hipErrorInvalidValue;
    // the strip kernels address activations and one expert matrix with 32-bit byte offsets
    if (uint64_t(a.T) * a.H * 2 >= (1ull << 32) || uint64_t(a.H) * a.F * 2 >= (1ull << 31)) return hipErrorInvalidValue;
    mark(2, 1);
    if (a.m_tile == 16) hipLaunchKernelGGL(gemm1_swiglu_kernel<1>, g1, dim3(256), 0, stream, a);
    else if (a.m_tile == 32) hipLaunchKernelGGL(gemm1_swiglu_kernel<2>, g1, dim3(256), 0, stream, a);
    else if (a.m_tile == 64) hipLaunchKernelGGL(gemm1_swiglu_kernel<4>, g1, dim3(256), 0, stream, a);
    else if (a.m_tile == 96) hipLaunchKernelGGL(gemm1_swiglu_kernel<6>, g1, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(gemm1_swiglu_kernel<8>, g1, dim3(256), 0, stream, a);
    mark(2, 0);
    mark(3, 1);
    if (a.m_tile == 16) hipLaunchKernelGGL(gemm2_kernel<1>, g2, dim3(256), 0, stream, a);
    else if (a.m_tile == 32) hipLaunchKernelGGL(gemm2_kernel<2>, g2, dim3(256), 0, stream, a);
    else if (a.m_tile == 64) hipLaunchKernelGGL(gemm2_kernel<4>, g2, dim3(256), 0, stream, a);
    else if (a.m_tile == 96) hipLaunchKernelGGL(gemm2_kernel<6>, g2, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(gemm2_kernel<8>, g2, dim3(256), 0, stream, a);
    mark(3, 0);
    const dim3 gc((a.H / 4 + 255) / 256, a.T, 1);
    mark(4, 1);
    launch_combine(gc);
    mark(4, 0);
    return hipGetLastError();
}

}  // namespace fluxmoe
