// Device-side structures and kernel launchers of libfluxmoe.so.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace fluxmoe {

constexpr uint32_t kHeaderBytes = 136;   // n, e0, sub_bits[64]
constexpr uint32_t kSubStreams = 64;
constexpr uint32_t kGroup = 64;          // block element counts are multiples of this
constexpr uint32_t kLutBits = 12;        // decode tables index 12 stream bits
constexpr uint32_t kLutEntries = 1u << kLutBits;

#if defined(__HIPCC__)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) u32x4 global_u32x4;
// Streaming (non-temporal) 16-byte accesses to device memory: data that is touched once.
// The pointers are cast to the global address space so that global_load / global_store are
// emitted instead of flat accesses.
__device__ __forceinline__ uint4 load_stream16(const void* p) {
    const u32x4 v = __builtin_nontemporal_load((const global_u32x4*)(uintptr_t)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream16(void* p, const uint4& v) {
    const u32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (global_u32x4*)(uintptr_t)p);
}
#endif

// One contiguous run of blocks of one tensor, decoded into one slot.
struct DecodeJob {
    uint64_t src;           // address of the run's first block (device memory)
    uint64_t dst;           // address of the tensor's first element in its slot
    uint32_t first_block;   // index of the run's first block in this type's block list
    uint32_t n_blocks;
    uint32_t tensor_elems;  // elements of the whole tensor (bounds every write)
    uint32_t pad;
};
static_assert(sizeof(DecodeJob) == 32, "DecodeJob layout");

// Header of a command buffer; the job lists and page-table updates follow it.
struct DecodeCmd {
    uint32_t n_jobs[2];        // [0] type 1 (gate/up), [1] type 2 (down)
    uint32_t total_blocks[2];
    uint32_t n_pt_updates;
    uint32_t pad[3];
};
static_assert(sizeof(DecodeCmd) == 32, "DecodeCmd layout");

// A small command buffer travels inside the kernel arguments (no separate upload, which costs a copy
// and a dependency in front of the kernel); kernel arguments are limited to 4 KiB in all.
constexpr uint32_t kInlineCmdBytes = 3584;

struct DecodeArgs {
    const DecodeCmd* cmd;        // device; ignored when inline_cmd is set
    uint32_t jobs_offset[2];     // byte offsets of the two job lists from the command header
    uint32_t upd_offset;         // byte offset of the int2 (index, value) page-table updates
    uint32_t wg_split;           // workgroups [0, wg_split) decode type 2, the rest type 1
    uint32_t apply_updates;      // non-zero: workgroup 0 applies the page-table updates
    uint32_t inline_cmd;         // non-zero: the command buffer is inline_words below
    const uint32_t* lut[2];      // device decode tables, [0] type 1, [1] type 2
    int32_t* page_table;         // device
    uint32_t* error_word;        // device
    uint32_t inline_words[kInlineCmdBytes / 4];
};
static_assert(sizeof(DecodeArgs) <= 4096 - 256, "kernel arguments must stay under 4 KiB with room for the hidden ones");

// Page-table updates small enough to travel inside the kernel arguments.
constexpr uint32_t kInlineUpdates = 448;
struct InlineUpdates {
    int32_t* page_table;
    uint32_t n;
    uint32_t pad;
    int32_t upd[2 * kInlineUpdates];   // (index, value) pairs
};

hipError_t launch_decode(const DecodeArgs& args, uint32_t n_workgroups, int waves_per_wg,
                         hipStream_t stream);
hipError_t launch_fill_i32(int32_t* p, int32_t v, uint64_t n, hipStream_t stream);
hipError_t launch_stream_copy(void* dst, const void* src, uint64_t bytes, uint32_t n_workgroups,
                              hipStream_t stream);
// page_table[upd[i].x] = upd[i].y for i < n (upd: device int2 list)
hipError_t launch_apply_updates(int32_t* page_table, const void* upd, uint32_t n, hipStream_t stream);
// the same with the (index, value) pairs read from host memory now and carried in the kernel arguments; n <= kInlineUpdates
hipError_t launch_apply_updates_inline(int32_t* page_table, const int32_t* host_upd, uint32_t n, hipStream_t stream);

// ---------------------------------------------------------------- expert FFN
struct FfnArgs {
    const uint16_t* tokens;      // BF16 [T][H]
    const int32_t* topk_ids;     // [T][K]
    const float* topk_w;         // [T][K]
    const int32_t* page_table;   // this layer's row: [n_experts]
    const uint16_t* slots13;     // type-1 arena
    const uint16_t* slots2;      // type-2 arena
    float* out;                  // [T][H]
    uint32_t T, K, H, F, E;
    uint32_t flags;
    // workspace carve-up (device)
    int32_t* expert_count;       // [E + 1]
    int32_t* expert_offset;      // [E + 2]
    int32_t* sorted_pair;        // [pairs_cap]  pair index (t * K + k), grouped by expert
    int32_t* pair_pos;           // [pairs_cap]  position of a pair in sorted order, -1 = skipped
    int4* tile_rec;              // [tiles_cap]  (expert, first sorted row, rows, slot); rows = 0 past the last tile
    int32_t* n_tiles;            // [1]
    uint16_t* hbuf;              // BF16 [pairs_cap][F]
    float* ybuf;                 // FP32 [ksplit][pairs_cap][H]
    uint32_t* error_word;
    uint32_t pairs_cap, tiles_cap, m_tile, ksplit;
    uint32_t tiled_waves;        // variant of the LDS-tiled kernels (m_tile 256): 2 LDS-direct loads, 8 or 4
                                 // wavefronts with register-staged loads
    uint32_t tiled_persist;      // LDS-direct kernels: workgroups per CU-sized round that walk through the tiles (1 = 256
                                 // workgroups), 0 = one workgroup per tile
    uint32_t tiled_total;        // set per launch by launch_ffn: tile numbers of the LDS-direct kernel's launch
    uint32_t tiled_group;        // super-rows of the LDS-direct gate/up kernel that share a column block in time;
                                 // 0 = launch_ffn derives it from the rows per expert
};

// hook(user, kind, begin, stream) is called around every kernel when timing is on
// (kinds: 1 grouping, 2 gate/up product + SwiGLU, 3 down product, 4 combine)
typedef void (*SpanHook)(void* user, int kind, int begin, hipStream_t stream);
hipError_t launch_ffn(const FfnArgs& args, int n_cus, hipStream_t stream, SpanHook hook, void* user);
hipError_t launch_mfma_probe(const void* operands, float* out, uint32_t n_workgroups, uint32_t iters,
                             hipStream_t stream);

}  // namespace fluxmoe
