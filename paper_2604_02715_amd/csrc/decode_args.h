// Device-side structures and launchers of the decode (materialization) kernels of libfluxmoe.so.
// bench.py keys the recorded HBM-traffic counters of the decode kernel to a hash of this file and
// decode_kernel.hip: nothing that the decode kernel does not compile from belongs here.
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

}  // namespace fluxmoe
