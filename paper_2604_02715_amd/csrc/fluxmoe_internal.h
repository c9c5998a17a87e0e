// Internal declarations shared by the host-side sources of libfluxmoe.so.
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "fluxmoe.h"
#include "kernels.h"

namespace fluxmoe {

int set_error(int status, const char* fmt, ...);

// Optimal prefix-code lengths limited to lmax for a 256-symbol histogram.
void limited_code_lengths(const uint64_t hist[256], uint32_t lmax, uint8_t lens[256]);
// Canonical codes for the lengths; codes[s] is read most significant bit first.
void canonical_codes(const uint8_t lens[256], uint16_t codes[256]);

struct TensorMeta {
    uint64_t first_block = 0;            // index in the layer blob
    std::vector<uint32_t> first_elem;    // [n_blocks + 1]
    uint64_t n_blocks() const { return first_elem.empty() ? 0 : first_elem.size() - 1; }
    // tier backing, set by fluxmoe_bind_layer and changed by fluxmoe_set_tensor_backing:
    // the tensor's blocks [0, n_host) are read from host_src, the rest from hbm_src
    uint64_t n_host = 0;
    const uint8_t* host_src = nullptr;   // pinned address of the tensor's block 0
    const uint8_t* hbm_src = nullptr;    // device address of the tensor's block n_host
    // uncompressed host backing (the CPU offload backend as Sec. 4.2 states it): pinned address of
    // the tensor's dense BF16 bytes; when set, n_host = 0 and hbm_src = nullptr
    const uint8_t* raw_src = nullptr;
    bool on_host() const { return n_host != 0 || raw_src != nullptr; }
};

struct LayerMeta {
    bool encoded = false;
    uint8_t lens[2][256];                // [0] type 1 (gate/up), [1] type 2 (down)
    uint64_t payload_bits[2] = {0, 0};
    std::vector<TensorMeta> tensors[2];  // per expert
    uint64_t n_blocks = 0;
    // tier binding
    bool bound = false;
    const uint8_t* hbm = nullptr;        // device pointer to block n_host_blocks
    const uint8_t* host = nullptr;       // pinned pointer to block 0
    uint64_t n_host_blocks = 0;
    uint64_t host_tensors = 0;           // tensors with n_host > 0
};

// Encode one flat tensor into consecutive blocks at dst (plan must come from plan_tensor).
void plan_tensor(const uint16_t* w, uint64_t n_elems, const uint8_t lens[256],
                 uint32_t block_bytes, std::vector<uint32_t>& first_elem);
void encode_tensor(const uint16_t* w, const std::vector<uint32_t>& first_elem,
                   const uint8_t lens[256], const uint16_t codes[256], uint32_t block_bytes,
                   uint8_t* dst);

}  // namespace fluxmoe
