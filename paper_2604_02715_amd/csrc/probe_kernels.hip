// Measurement aid of libfluxmoe.so: the decode kernel's memory traffic with none of its work.
// Nothing here is on the materialization path.
#include "decode_args.h"
#include "kernels.h"

namespace fluxmoe {
namespace {

// Output bytes of block nb and of all blocks before it.  Real blocks decode to a multiple of 128
// bytes that varies with their content; here three blocks of every eight write `small + 128`
// bytes and the others `small`, so that consecutive blocks stay contiguous in the output, every
// piece starts on a 128-byte line and the mean can be set to a pool's dense / compressed ratio.
constexpr uint32_t kLargeMask = 0x49;     // blocks 0, 3 and 6 of every eight
__device__ __forceinline__ uint64_t out_offset(uint32_t nb, uint32_t small) {
    const uint32_t r = nb & 7u;
    return uint64_t(nb >> 3) * (8ull * small + 3 * 128) + uint64_t(r) * small +
           128u * uint32_t(__builtin_popcount(kLargeMask & ((1u << r) - 1u)));
}

// The launch shape and the accesses of decode_kernel: workgroups of WAVES wavefronts, blocks dealt
// round-robin over all wavefronts of the grid, a wavefront reads its 4 KiB block with four streaming
// 16-byte loads per lane and writes the block's output in contiguous pieces of 1 KiB with streaming
// 16-byte stores.  What is stored depends on what was loaded, so a block's stores wait for its loads
// as they do in the decoder.
// order 0: as the decode kernel (a wavefront's blocks are a whole grid of wavefronts apart); 1: a workgroup
// covers WAVES * per_wave consecutive blocks, its wavefronts passing over them side by side; 2: a wavefront
// covers per_wave consecutive blocks.
template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void stream_mix_kernel(const char* __restrict__ src, char* __restrict__ dst,
                                                               uint32_t n_blocks, uint32_t small, uint32_t per_wave,
                                                               uint32_t order) {
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t n_waves = gridDim.x * WAVES;
    uint32_t first = blockIdx.x * WAVES + wave, step = n_waves, end = n_blocks;
    if (order == 1) {
        first = blockIdx.x * WAVES * per_wave + wave;
        step = WAVES;
        end = min(n_blocks, (blockIdx.x + 1) * WAVES * per_wave);
    } else if (order == 2) {
        first = (blockIdx.x * WAVES + wave) * per_wave;
        step = 1;
        end = min(n_blocks, first + per_wave);
    }
    for (uint32_t nb = first; nb < end; nb += step) {
        const char* s = src + uint64_t(nb) * 4096 + 16 * lane;
        const uint4 v0 = load_stream16(s);
        const uint4 v1 = load_stream16(s + 1024);
        const uint4 v2 = load_stream16(s + 2048);
        const uint4 v3 = load_stream16(s + 3072);
        uint4 o = make_uint4(v0.x ^ v1.x ^ v2.x ^ v3.x, v0.y ^ v1.y ^ v2.y ^ v3.y, v0.z ^ v1.z ^ v2.z ^ v3.z,
                             v0.w ^ v1.w ^ v2.w ^ v3.w);
        const uint32_t bytes = small + (((kLargeMask >> (nb & 7u)) & 1u) ? 128u : 0u);
        char* d = dst + out_offset(nb, small);
        for (uint32_t off = 16 * lane; off < bytes; off += 1024) {
            store_stream16(d + off, o);
            o.x += 1u;
        }
    }
}

}  // namespace

uint64_t stream_mix_out_bytes(uint64_t n_blocks, uint32_t small) {
    uint64_t total = (n_blocks >> 3) * (8ull * small + 3 * 128);
    for (uint32_t r = 0; r < (n_blocks & 7u); ++r) total += small + (((kLargeMask >> r) & 1u) ? 128u : 0u);
    return total;
}

hipError_t launch_stream_mix(void* dst, const void* src, uint32_t n_blocks, uint32_t small, int waves_per_wg,
                             uint32_t per_wave, uint32_t order, uint32_t n_workgroups, hipStream_t stream) {
    const char* s = static_cast<const char*>(src);
    char* d = static_cast<char*>(dst);
    // the decode kernel's LDS footprint (a staged block per wavefront and one table), unused here, so that as
    // many workgroups share a CU as there
    const size_t lds = size_t(waves_per_wg) * 4096 + 4 * kLutEntries;
    switch (waves_per_wg) {
        case 4: hipLaunchKernelGGL(stream_mix_kernel<4>, dim3(n_workgroups), dim3(256), lds, stream, s, d, n_blocks, small, per_wave, order); break;
        case 8: hipLaunchKernelGGL(stream_mix_kernel<8>, dim3(n_workgroups), dim3(512), lds, stream, s, d, n_blocks, small, per_wave, order); break;
        case 16: hipLaunchKernelGGL(stream_mix_kernel<16>, dim3(n_workgroups), dim3(1024), lds, stream, s, d, n_blocks, small, per_wave, order); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace fluxmoe
