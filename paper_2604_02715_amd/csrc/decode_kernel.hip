// Decode + paged scatter kernel (gfx950).
//
// Reconstructs dense BF16 expert weights from the compressed pool (paper Sec. 4.2
// "Compressed GPU backend", Sec. 5 "Expert memory backends": exponent bits Huffman coded,
// sign/mantissa raw) straight into the staging slots the page table points at (Sec. 4.1
// "PagedTensor": materialization updates block contents).
//
// Work decomposition: one 64-lane wavefront decodes one 4 KiB block at a time.  The block
// (32 full 128-byte lines) is read with coalesced 16-byte loads and parked in LDS; the
// decode table of the tensor type sits in LDS once per workgroup.  Lane j owns sub-stream
// j: its start bit comes from a wavefront prefix sum over the 64 sub-stream bit lengths in
// the block header.  Elements are dealt to lanes in runs of 8, so after every 8 symbols a
// lane holds 16 contiguous output bytes and the wavefront writes 1 KiB of contiguous,
// 128-byte aligned slot memory.  Output positions are static; only bit positions are data
// dependent.
//
// Symbols are decoded two at a time.  A lane keeps the bit position of its sub-stream and the two
// stream words around it in registers; per pair it funnel-shifts them into a 32-bit window
// (v_alignbit_b32) and looks the next 12 stream bits up in a pair table: an entry holds the exponent
// fields of the next two symbols, already in their BF16 positions of a packed pair of outputs, and
// the sum of their code lengths.  The stream word after the two held ones is read together with the
// table entry, so a pair costs one LDS round trip.  If the two codes do not fit into 12 bits together
// (under 1 % of the pairs on weight-like data) the entry holds the first symbol only and is marked;
// the marked lanes take a second lookup.
// Entry layout: bits 0..5 bits to advance, 7..14 first exponent, 15..18 length of the first code,
// 23..30 second exponent, 31 = only the first symbol is valid.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstring>

#include "decode_args.h"

namespace fluxmoe {

namespace {

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (no LDS round trips):
// four shifted adds inside each row of 16 lanes, then the totals of rows 0 and 2 go to rows 1 and
// 3, then the total of the first half to the second half.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    // update_dpp(old, src, ctrl, row_mask, bank_mask, bound_ctrl): lanes that receive nothing keep `old` (0)
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x111, 0xF, 0xF, false));   // row_shr:1
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x112, 0xF, 0xF, false));   // row_shr:2
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x114, 0xF, 0xF, false));   // row_shr:4
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x118, 0xF, 0xF, false));   // row_shr:8
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x142, 0xA, 0xF, false));   // row_bcast:15 -> rows 1, 3
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x143, 0xC, 0xF, false));   // row_bcast:31 -> rows 2, 3
    return v;
}

constexpr uint32_t kPairExpMask = 0x7F807F80u;     // the two exponent fields of an entry
constexpr uint32_t kLutByteMask = (kLutEntries - 1) << 2;

// (w & mask) | base in one instruction: byte offset of a table entry from the window w, whose bits
// 2..13 are the 12 stream bits to look up (positions are kept minus 2 for that); the compiler emits two
// instructions because both constants are literals
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask_sgpr, uint32_t base_vgpr) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask_sgpr), "v"(base_vgpr));
    return r;
}

// Per-lane stream state.  p: the lane's bit position counted from LDS byte 0 (the staged block's LDS
// address times 8 is folded in; it is a multiple of 32, so word address and bit offset come out of the
// same register), minus 2.  ka = (p / 32) * 4 is the LDS byte address of the stream word that holds
// bit p; w0, w1 are that word and the next one.
struct Stream {
    uint32_t p, ka, w0, w1;
};

// Decode the next two symbols.  The table lookup and the read of the stream word after w1 are issued
// together, so a pair costs one LDS round trip: a pair advances the position by 24 bits at most, so
// the next pair's two words are among w0, w1 and that third word.
__device__ __forceinline__ uint32_t decode_pair(const uint8_t* __restrict__ lds0, uint32_t lut_mask, uint32_t lut_base,
                                                Stream& st) {
    const uint32_t w = __builtin_amdgcn_alignbit(st.w1, st.w0, st.p);     // stream bits from position p on
    uint32_t e = *reinterpret_cast<const uint32_t*>(lds0 + and_or(w, lut_mask, lut_base));
    const uint32_t w2 = *reinterpret_cast<const uint32_t*>(lds0 + st.ka + 8);
    if (int32_t(e) < 0) {                                                 // rare: the two codes exceed 12 bits
        const uint32_t l0 = e & 63u;
        const uint32_t e2 = *reinterpret_cast<const uint32_t*>(lds0 + and_or(w >> l0, lut_mask, lut_base));
        e = (e & 0x7F80u) | ((e2 & 0x7F80u) << 16) | (l0 + ((e2 >> 15) & 15u));
    }
    st.p += e & 63u;
    const uint32_t ka = (st.p >> 3) & ~3u;
    const bool adv = ka != st.ka;
    st.w0 = adv ? st.w1 : st.w0;
    st.w1 = adv ? w2 : st.w1;
    st.ka = ka;
    return e;                     // the caller keeps the exponent fields only (kPairExpMask)
}

__device__ __forceinline__ uint32_t join_pair(uint32_t entry, uint32_t sm4, uint32_t sel) {
    // spread two raw bytes into two 16-bit lanes [s, s]; exponent bits from the entry, sign and mantissa
    // from the raw bytes (one v_bfi_b32)
    const uint32_t t = __builtin_amdgcn_perm(sm4, sm4, sel);
    return (entry & kPairExpMask) | (t & ~kPairExpMask);
}

// Job records are read through the scalar data path (they are uniform over the wavefront and are
// not written while the kernel runs): a vector load would have to wait for the stores in flight.
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ DecodeJob load_job(const DecodeJob* jobs, uint32_t j) {
    const DecodeJob* ptr = jobs + j;
    u32x8 v;
    asm volatile("s_load_dwordx8 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(ptr) : "memory");
    DecodeJob job;
    job.src = uint64_t(v[0]) | (uint64_t(v[1]) << 32);
    job.dst = uint64_t(v[2]) | (uint64_t(v[3]) << 32);
    job.first_block = v[4];
    job.n_blocks = v[5];
    job.tensor_elems = v[6];
    job.pad = v[7];
    return job;
}

// The job whose block range contains block b (jobs are ascending and cover [0, total) without gaps).
// Tensors of one type have almost the same number of blocks, so the proportional guess is off by a
// job or two at most; the scans correct it.
__device__ __forceinline__ DecodeJob find_job(const DecodeJob* jobs, uint32_t n_jobs, uint32_t total, uint32_t b) {
    uint32_t j = uint32_t(uint64_t(b) * n_jobs / total);
    DecodeJob job = load_job(jobs, j);
    while (b < job.first_block) job = load_job(jobs, --j);
    while (b >= job.first_block + job.n_blocks) job = load_job(jobs, ++j);
    return job;
}

constexpr int kBlockBytes = 4096;
constexpr int kBlockWords = kBlockBytes / 4;

// Decode the block staged at `stage` into its place in the slot.  A block that fails validation is
// skipped and flagged.
__device__ __forceinline__ void decode_block(const uint32_t* __restrict__ stage, const uint8_t* __restrict__ lds0,
                                                 uint32_t lut_mask, uint32_t lut_base, const DecodeJob& job,
                                                 uint32_t* error_word, int lane) {
    const uint32_t n = __builtin_amdgcn_readfirstlane(stage[0]);
    const uint32_t e0 = __builtin_amdgcn_readfirstlane(stage[1]);
    const uint32_t sb = reinterpret_cast<const uint16_t*>(stage)[4 + lane];
    const uint32_t incl = wave_inclusive_scan(sb);
    const uint32_t total_bits = __builtin_amdgcn_readlane(incl, 63);
    const bool ok = n != 0 && (n & 63u) == 0 && n <= uint32_t(kBlockBytes) - kHeaderBytes &&
                    uint64_t(e0) + n <= job.tensor_elems && (e0 & 63u) == 0 &&
                    (kHeaderBytes + n) * 8u + total_bits <= uint32_t(kBlockBytes) * 8u;
    if (!ok) {
        if (lane == 0) atomicOr(error_word, 1u);
        return;
    }
    // first bit of this lane's sub-stream, minus 2, counted from LDS byte 0
    Stream st;
    st.p = (kHeaderBytes + n) * 8u + (incl - sb) - 2u + 8u * uint32_t(reinterpret_cast<const uint8_t*>(stage) - lds0);
    st.ka = (st.p >> 3) & ~3u;
    st.w0 = *reinterpret_cast<const uint32_t*>(lds0 + st.ka);
    st.w1 = *reinterpret_cast<const uint32_t*>(lds0 + st.ka + 4);
    const uint32_t n_runs = n >> 3;
    uint16_t* out = reinterpret_cast<uint16_t*>(job.dst) + e0;
    for (uint32_t r = lane; r < n_runs; r += 64) {
        const uint32_t sm_lo = stage[kHeaderBytes / 4 + 2 * r];
        const uint32_t sm_hi = stage[kHeaderBytes / 4 + 2 * r + 1];
        uint4 o;
        const uint32_t x0 = decode_pair(lds0, lut_mask, lut_base, st);
        o.x = join_pair(x0, sm_lo, 0x01010000u);
        const uint32_t x1 = decode_pair(lds0, lut_mask, lut_base, st);
        o.y = join_pair(x1, sm_lo, 0x03030202u);
        const uint32_t x2 = decode_pair(lds0, lut_mask, lut_base, st);
        o.z = join_pair(x2, sm_hi, 0x01010000u);
        const uint32_t x3 = decode_pair(lds0, lut_mask, lut_base, st);
        o.w = join_pair(x3, sm_hi, 0x03030202u);
        store_stream16(out + 8u * r, o);
    }
}

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void decode_kernel(DecodeArgs a) {
    // the staged blocks first, the table behind them: the word a window read takes past the end of the
    // last staged block is then a table word (unused bits) and no padding is needed
    __shared__ __align__(16) uint32_t lds_all[WAVES * kBlockWords + kLutEntries];
    uint32_t* const lut = lds_all + WAVES * kBlockWords;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the command buffer: in device memory, or - when small - inside the kernel arguments, which are read in
    // place through the kernel-argument segment's address (taking the address of `a`'s member would copy it)
    const DecodeCmd* cmd = a.cmd;
    if (a.inline_cmd)
        cmd = reinterpret_cast<const DecodeCmd*>(reinterpret_cast<const char*>((const void*)__builtin_amdgcn_kernarg_segment_ptr()) +
                                                 offsetof(DecodeArgs, inline_words));

    // page-table updates ride along with the first workgroup
    if (blockIdx.x == 0 && a.apply_updates) {
        const uint32_t n_upd = cmd->n_pt_updates;
        const int2* upd = reinterpret_cast<const int2*>(reinterpret_cast<const char*>(cmd) +
                                                        a.upd_offset);
        for (uint32_t i = tid; i < n_upd; i += WAVES * 64) a.page_table[upd[i].x] = upd[i].y;
    }

    const int type = (blockIdx.x < a.wg_split) ? 1 : 0;   // type-2 (down) list first
    const uint32_t wg_first = type ? 0u : a.wg_split;
    const uint32_t wg_count = type ? a.wg_split : (gridDim.x - a.wg_split);
    const uint32_t total = __builtin_amdgcn_readfirstlane(cmd->total_blocks[type]);
    const uint32_t n_jobs = __builtin_amdgcn_readfirstlane(cmd->n_jobs[type]);
    const DecodeJob* jobs = reinterpret_cast<const DecodeJob*>(
        reinterpret_cast<const char*>(cmd) + a.jobs_offset[type]);

    {   // decode table of this tensor type -> LDS
        const uint4* src = reinterpret_cast<const uint4*>(a.lut[type]);
        uint4* dst = reinterpret_cast<uint4*>(lut);
        for (int i = tid; i < int(kLutEntries / 4); i += WAVES * 64) dst[i] = src[i];
    }
    __syncthreads();

    // Blocks are dealt round-robin over all wavefronts of this tensor type, and the grid holds many
    // more workgroups than fit on the chip at once: at any moment the running wavefronts work on one
    // contiguous window of the pool and of the slots (which HBM serves better than thousands of
    // far-apart sequential streams), and a CU whose wavefronts are served slowly simply takes fewer
    // workgroups (the arbitration between wavefronts is not fair: with one long-lived wavefront per
    // share of the blocks the slowest one takes twice as long as the fastest).
    const uint32_t n_waves = wg_count * WAVES;
    uint32_t nb = (blockIdx.x - wg_first) * WAVES + wave;
    if (nb >= total) return;

    uint32_t* stage = lds_all + wave * kBlockWords;
    uint4* st4 = reinterpret_cast<uint4*>(stage);
    const uint8_t* lds0 = reinterpret_cast<const uint8_t*>(lds_all);
    // mask (scalar register) and base (vector register) of a table address, so that the address is one
    // v_and_or_b32 (an instruction takes one literal or one scalar register at most)
    uint32_t lut_mask, lut_base;
    asm volatile("s_mov_b32 %0, %2\n\tv_mov_b32 %1, %3" : "=s"(lut_mask), "=v"(lut_base) : "n"(kLutByteMask), "n"(WAVES * kBlockBytes));
    DecodeJob job = find_job(jobs, n_jobs, total, nb);
    for (;;) {
        const char* src = reinterpret_cast<const char*>(job.src + uint64_t(nb - job.first_block) * kBlockBytes) + 16 * lane;
        const uint4 v0 = load_stream16(src);
        const uint4 v1 = load_stream16(src + 1024);
        const uint4 v2 = load_stream16(src + 2048);
        const uint4 v3 = load_stream16(src + 3072);
        // LDS operations of one wavefront complete in order; the staged block is private to it, and
        // everything read from the previous block has been consumed
        st4[lane] = v0;
        st4[lane + 64] = v1;
        st4[lane + 128] = v2;
        st4[lane + 192] = v3;
        decode_block(stage, lds0, lut_mask, lut_base, job, a.error_word, lane);
        const uint32_t after = nb + n_waves;
        if (after >= total || after <= nb) break;          // uniform
        nb = after;
        if (nb >= job.first_block + job.n_blocks) job = find_job(jobs, n_jobs, total, nb);
    }
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& args, uint32_t n_workgroups, int waves_per_wg, hipStream_t stream) {
    switch (waves_per_wg) {
        case 4: hipLaunchKernelGGL(decode_kernel<4>, dim3(n_workgroups), dim3(256), 0, stream, args); break;
        case 8: hipLaunchKernelGGL(decode_kernel<8>, dim3(n_workgroups), dim3(512), 0, stream, args); break;
        case 16: hipLaunchKernelGGL(decode_kernel<16>, dim3(n_workgroups), dim3(1024), 0, stream, args); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ small helpers
namespace {
__global__ void fill_i32_kernel(int32_t* p, int32_t v, uint64_t n) {
    const uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
}  // namespace

namespace {
__global__ void apply_updates_kernel(int32_t* page_table, const int2* upd, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) page_table[upd[i].x] = upd[i].y;
}
}  // namespace

namespace {
__global__ void apply_updates_inline_kernel(InlineUpdates u) {
    const int2* upd = reinterpret_cast<const int2*>(reinterpret_cast<const char*>((const void*)__builtin_amdgcn_kernarg_segment_ptr()) +
                                                    offsetof(InlineUpdates, upd));
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < u.n) u.page_table[upd[i].x] = upd[i].y;
}
}  // namespace

hipError_t launch_apply_updates_inline(int32_t* page_table, const int32_t* host_upd, uint32_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    if (n > kInlineUpdates) return hipErrorInvalidValue;
    InlineUpdates u;
    u.page_table = page_table;
    u.n = n;
    u.pad = 0;
    std::memcpy(u.upd, host_upd, size_t(n) * 8);
    hipLaunchKernelGGL(apply_updates_inline_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, u);
    return hipGetLastError();
}

hipError_t launch_apply_updates(int32_t* page_table, const void* upd, uint32_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(apply_updates_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, page_table,
                       static_cast<const int2*>(upd), n);
    return hipGetLastError();
}

namespace {
// Plain streaming copy with the same 16-byte non-temporal accesses the decode kernel uses:
// the reference point for achievable HBM bandwidth and for hardware-counter calibration.
__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src,
                                                          uint4* __restrict__ dst, uint64_t n16) {
    const uint64_t stride = uint64_t(gridDim.x) * 256;
    for (uint64_t i = uint64_t(blockIdx.x) * 256 + threadIdx.x; i < n16; i += stride)
        store_stream16(dst + i, load_stream16(src + i));
}
}  // namespace

hipError_t launch_stream_copy(void* dst, const void* src, uint64_t bytes, uint32_t n_workgroups,
                              hipStream_t stream) {
    if (bytes < 16) return hipSuccess;
    hipLaunchKernelGGL(stream_copy_kernel, dim3(n_workgroups), dim3(256), 0, stream,
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
    return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* p, int32_t v, uint64_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_i32_kernel, dim3(uint32_t((n + 255) / 256)), dim3(256), 0, stream, p, v, n);
    return hipGetLastError();
}

}  // namespace fluxmoe
