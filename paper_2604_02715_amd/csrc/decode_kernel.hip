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
// j: its start bit comes from a wavefront exclusive prefix sum over the 64 sub-stream bit
// lengths in the block header.  Elements are dealt to lanes in runs of 8, so after every 8
// symbols a lane holds 16 contiguous output bytes and the wavefront writes 1 KiB of
// contiguous, 128-byte aligned slot memory.  Output positions are static; only bit
// positions are data dependent.
//
// Each lane keeps the unread bits of its sub-stream in a 64-bit reservoir that is topped up
// from the staged block one 32-bit word at a time, only by the lanes that have run low, so
// every stream word is fetched from LDS once.  Per symbol the lane looks the reservoir's low
// 12 bits up in the table (-> exponent field + length) and shifts the reservoir by the length.
// Table entries are (exponent << 23) | length: shifting by an entry uses only its low bits,
// adding entries accumulates lengths in the low bits, and the high half of an entry is the
// exponent already in BF16 position.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace fluxmoe {

namespace {

constexpr int kBlockWords = 1024;          // 4 KiB block
constexpr int kStageWords = kBlockWords + 4;  // + padding for the window's second word

__device__ __forceinline__ uint32_t wave_exclusive_scan(uint32_t v, int lane) {
    uint32_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    return incl - v;
}

// Per-lane bit reservoir: `buf` holds the unread bits of the lane's sub-stream with the next
// stream bit at bit kShift (the two bits below are don't-care, so a table byte address is one
// AND away); `cnt` counts valid bits; `k` is the index of the next stream word in the staged
// block.  Every stream word is fetched from LDS exactly once, and only by the lanes that have
// run low, which keeps the fetches sparse and mostly free of bank conflicts.
constexpr uint32_t kShift = 2;
constexpr uint32_t kRefillBelow = 25;   // a pair needs at most 24 bits; 24 + 32 + kShift <= 64

struct Reservoir {
    uint64_t buf;
    uint32_t cnt;
    uint32_t k;
};

// Decode one pair of symbols; returns the two exponent fields packed as BF16 halves.
__device__ __forceinline__ uint32_t decode_pair(const uint32_t* __restrict__ stage,
                                                const uint32_t* __restrict__ lut, Reservoir& r) {
    if (r.cnt < kRefillBelow) {
        const uint64_t w = stage[r.k & (kBlockWords - 1)];
        r.buf |= w << (r.cnt + kShift);
        r.cnt += 32;
        r.k += 1;
    }
    const uint32_t e0 = lut[(uint32_t(r.buf) >> kShift) & (kLutEntries - 1)];
    r.buf >>= (e0 & 63u);
    const uint32_t e1 = lut[(uint32_t(r.buf) >> kShift) & (kLutEntries - 1)];
    r.buf >>= (e1 & 63u);
    r.cnt -= (e0 + e1) & 31u;
    // bytes: [e0.b2, e0.b3, e1.b2, e1.b3]
    return __builtin_amdgcn_perm(e1, e0, 0x07060302u);
}

__device__ __forceinline__ uint32_t join_pair(uint32_t exps, uint32_t sm4, uint32_t sel) {
    // spread two raw bytes into two 16-bit lanes [s, s] and keep mantissa low / sign high
    const uint32_t t = __builtin_amdgcn_perm(sm4, sm4, sel);
    return (t & 0x807F807Fu) | exps;
}

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void decode_kernel(DecodeArgs a) {
    __shared__ uint32_t lut[kLutEntries];
    __shared__ uint32_t stage_all[WAVES][kStageWords];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const DecodeCmd* cmd = a.cmd;

    // page-table updates ride along with the first workgroup
    if (blockIdx.x == 0) {
        const uint32_t n_upd = cmd->n_pt_updates;
        const int2* upd = reinterpret_cast<const int2*>(reinterpret_cast<const char*>(cmd) +
                                                        a.upd_offset);
        for (uint32_t i = tid; i < n_upd; i += WAVES * 64) a.page_table[upd[i].x] = upd[i].y;
    }

    const int type = (blockIdx.x < a.wg_split) ? 1 : 0;   // type-2 (down) list first
    const uint32_t wg_first = type ? 0u : a.wg_split;
    const uint32_t wg_count = type ? a.wg_split : (gridDim.x - a.wg_split);
    const uint32_t total = cmd->total_blocks[type];
    const uint32_t n_jobs = cmd->n_jobs[type];
    const DecodeJob* jobs = reinterpret_cast<const DecodeJob*>(
        reinterpret_cast<const char*>(cmd) + a.jobs_offset[type]);

    {   // decode table of this tensor type -> LDS
        const uint4* src = reinterpret_cast<const uint4*>(a.lut[type]);
        uint4* dst = reinterpret_cast<uint4*>(lut);
        for (int i = tid; i < int(kLutEntries / 4); i += WAVES * 64) dst[i] = src[i];
    }
    __syncthreads();

    // Blocks are dealt to wavefronts in chunks of a.chunk_blocks, round-robin over all
    // wavefronts of this tensor type: at any moment the grid works on one contiguous window
    // of the pool and of the slots, which HBM serves better than thousands of far-apart
    // sequential streams.
    const uint32_t n_waves = wg_count * WAVES;
    const uint32_t my_wave = (blockIdx.x - wg_first) * WAVES + wave;
    const uint32_t chunk = a.chunk_blocks;
    if (uint64_t(my_wave) * chunk >= total) return;

    uint32_t j = 0;
    DecodeJob job = jobs[0];
    uint32_t* stage = stage_all[wave];
    for (uint64_t c0 = uint64_t(my_wave) * chunk; c0 < total; c0 += uint64_t(n_waves) * chunk) {
      const uint32_t b_end = uint32_t(min(uint64_t(total), c0 + chunk));
      uint32_t b = uint32_t(c0);
      if (b >= job.first_block + job.n_blocks) {
        // job that contains block b: last index with first_block <= b (jobs are ascending)
        uint32_t lo = j + 1, hi = n_jobs - 1;
        while (lo < hi) {
            const uint32_t mid = (lo + hi + 1) >> 1;
            if (jobs[mid].first_block <= b) lo = mid; else hi = mid - 1;
        }
        j = lo;
        job = jobs[j];
      }
      for (; b < b_end; ++b) {
        while (b >= job.first_block + job.n_blocks) job = jobs[++j];
        const char* src = reinterpret_cast<const char*>(job.src + uint64_t(b - job.first_block) * 4096u);
        const uint4 v0 = load_stream16(src + 16 * lane);
        const uint4 v1 = load_stream16(src + 16 * lane + 1024);
        const uint4 v2 = load_stream16(src + 16 * lane + 2048);
        const uint4 v3 = load_stream16(src + 16 * lane + 3072);
        uint4* st4 = reinterpret_cast<uint4*>(stage);
        st4[lane] = v0;
        st4[lane + 64] = v1;
        st4[lane + 128] = v2;
        st4[lane + 192] = v3;
        // LDS operations of one wavefront complete in order; the buffer is private to it

        const uint32_t n = stage[0];
        const uint32_t e0 = stage[1];
        const uint32_t sb = (stage[2 + (lane >> 1)] >> ((lane & 1) * 16)) & 0xFFFFu;
        const uint32_t start = wave_exclusive_scan(sb, lane);
        const uint32_t total_bits = __shfl(start + sb, 63, 64);
        const bool ok = n != 0 && (n & 63u) == 0 && n <= 4096u - kHeaderBytes &&
                        uint64_t(e0) + n <= job.tensor_elems && (e0 & 63u) == 0 &&
                        (kHeaderBytes + n) * 8u + total_bits <= 4096u * 8u;
        if (!ok) {
            if (lane == 0) atomicOr(a.error_word, 1u);
            continue;
        }
        const uint32_t p0 = (kHeaderBytes + n) * 8u + start;     // first bit of this lane's sub-stream
        Reservoir q;
        q.k = (p0 >> 5) + 1;
        q.cnt = 32u - (p0 & 31u);
        q.buf = uint64_t(stage[p0 >> 5] >> (p0 & 31u)) << kShift;
        const uint32_t n_runs = n >> 3;
        uint16_t* out = reinterpret_cast<uint16_t*>(job.dst) + e0;
        for (uint32_t r = lane; r < n_runs; r += 64) {
            const uint32_t sm_lo = stage[kHeaderBytes / 4 + 2 * r];
            const uint32_t sm_hi = stage[kHeaderBytes / 4 + 2 * r + 1];
            uint4 o;
            const uint32_t x0 = decode_pair(stage, lut, q);
            o.x = join_pair(x0, sm_lo, 0x01010000u);
            const uint32_t x1 = decode_pair(stage, lut, q);
            o.y = join_pair(x1, sm_lo, 0x03030202u);
            const uint32_t x2 = decode_pair(stage, lut, q);
            o.z = join_pair(x2, sm_hi, 0x01010000u);
            const uint32_t x3 = decode_pair(stage, lut, q);
            o.w = join_pair(x3, sm_hi, 0x03030202u);
            store_stream16(out + 8u * r, o);
        }
      }
    }
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& args, uint32_t n_workgroups, int waves_per_wg,
                         hipStream_t stream) {
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
