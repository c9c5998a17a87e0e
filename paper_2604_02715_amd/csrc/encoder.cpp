// Offline encoder of the compressed expert pool (host only).
//
// Paper Sec. 4.2 "Compressed GPU backend": only the exponent bits of the BF16 routed-expert
// weights are Huffman coded, offline; sign and mantissa bits are stored unchanged.  The
// block container is this library's own (documented in fluxmoe.h).
#include <algorithm>
#include <array>
#include <cstring>

#include "fluxmoe_internal.h"

namespace fluxmoe {

namespace {

struct Item {
    uint64_t weight;
    std::array<uint8_t, 256> count;   // how many leaves of each symbol the item contains
};

}  // namespace

// Package-merge: every used symbol contributes one leaf per level 1..lmax; from the deepest
// level upwards the items of a level (leaves plus the packages formed below) are sorted by
// weight and paired into packages for the level above; the 2(m-1) lightest items of level
// 1 are selected and a symbol's code length is the number of its leaves among them.
void limited_code_lengths(const uint64_t hist[256], uint32_t lmax, uint8_t lens[256]) {
    std::memset(lens, 0, 256);
    std::vector<int> used;
    for (int s = 0; s < 256; ++s)
        if (hist[s]) used.push_back(s);
    const size_t m = used.size();
    if (m == 0) return;
    if (m == 1) {
        lens[used[0]] = 1;
        return;
    }
    std::vector<Item> leaves(m);
    for (size_t i = 0; i < m; ++i) {
        leaves[i].weight = hist[used[i]];
        leaves[i].count.fill(0);
        leaves[i].count[used[i]] = 1;
    }
    auto by_weight = [](const Item& a, const Item& b) { return a.weight < b.weight; };
    std::stable_sort(leaves.begin(), leaves.end(), by_weight);
    std::vector<Item> packages, level;
    for (uint32_t depth = lmax; depth >= 1; --depth) {
        level.clear();
        level.resize(leaves.size() + packages.size());
        std::merge(leaves.begin(), leaves.end(), packages.begin(), packages.end(),
                   level.begin(), by_weight);
        if (depth == 1) break;
        packages.clear();
        for (size_t i = 0; i + 1 < level.size(); i += 2) {
            Item p;
            p.weight = level[i].weight + level[i + 1].weight;
            for (int s = 0; s < 256; ++s) p.count[s] = level[i].count[s] + level[i + 1].count[s];
            packages.push_back(p);
        }
    }
    const size_t take = 2 * (m - 1);
    for (size_t i = 0; i < take && i < level.size(); ++i)
        for (int s = 0; s < 256; ++s) lens[s] += level[i].count[s];
}

void canonical_codes(const uint8_t lens[256], uint16_t codes[256]) {
    std::memset(codes, 0, 256 * sizeof(uint16_t));
    uint32_t next = 0;
    uint32_t prev_len = 0;
    bool first = true;
    for (uint32_t len = 1; len <= 16; ++len) {
        for (int s = 0; s < 256; ++s) {
            if (lens[s] != len) continue;
            if (first) {
                next = 0;
                first = false;
            } else {
                next = (next + 1) << (len - prev_len);
            }
            codes[s] = static_cast<uint16_t>(next);
            prev_len = len;
        }
    }
}

static inline uint32_t exponent_of(uint16_t w) { return (w >> 7) & 0xFFu; }

// Greedy packing in groups of 64 elements: a block takes the largest number of whole groups
// whose header + raw bytes + code words still fit.
void plan_tensor(const uint16_t* w, uint64_t n_elems, const uint8_t lens[256],
                 uint32_t block_bytes, std::vector<uint32_t>& first_elem) {
    first_elem.clear();
    first_elem.push_back(0);
    uint64_t pos = 0;
    while (pos < n_elems) {
        uint64_t n = 0, bits = 0;
        while (pos + n < n_elems) {
            uint64_t gbits = 0;
            const uint16_t* g = w + pos + n;
            for (uint32_t i = 0; i < kGroup; ++i) gbits += lens[exponent_of(g[i])];
            const uint64_t need = kHeaderBytes + (n + kGroup) + 4 * ((bits + gbits + 31) / 32);
            if (need > block_bytes) break;
            n += kGroup;
            bits += gbits;
        }
        pos += n;   // n >= 64 always: 136 + 64 + 96 bytes fit any supported block size
        first_elem.push_back(static_cast<uint32_t>(pos));
    }
}

void encode_tensor(const uint16_t* w, const std::vector<uint32_t>& first_elem,
                   const uint8_t lens[256], const uint16_t codes[256], uint32_t block_bytes,
                   uint8_t* dst) {
    // codes with their first bit in bit 0 (the stream is filled from bit 0 upwards)
    uint32_t rev[256];
    for (int s = 0; s < 256; ++s) {
        uint32_t r = 0;
        for (uint32_t b = 0; b < lens[s]; ++b) r |= ((codes[s] >> (lens[s] - 1 - b)) & 1u) << b;
        rev[s] = r;
    }
    const size_t n_blocks = first_elem.size() - 1;
    for (size_t k = 0; k < n_blocks; ++k) {
        uint8_t* blk = dst + k * static_cast<size_t>(block_bytes);
        std::memset(blk, 0, block_bytes);
        const uint32_t e0 = first_elem[k];
        const uint32_t n = first_elem[k + 1] - e0;
        const uint16_t* src = w + e0;
        std::memcpy(blk, &n, 4);
        std::memcpy(blk + 4, &e0, 4);
        uint8_t* sm = blk + kHeaderBytes;
        for (uint32_t m = 0; m < n; ++m)
            sm[m] = static_cast<uint8_t>(((src[m] >> 8) & 0x80u) | (src[m] & 0x7Fu));
        // sub-streams are written one after another by a single bit writer
        uint8_t* area = blk + kHeaderBytes + n;
        uint64_t acc = 0;
        uint32_t fill = 0;
        size_t word = 0;
        const uint32_t n_runs = n / 8;
        for (uint32_t j = 0; j < kSubStreams; ++j) {
            uint32_t bits_j = 0;
            for (uint32_t r = j; r < n_runs; r += kSubStreams) {
                const uint16_t* run = src + 8u * r;
                for (uint32_t i = 0; i < 8; ++i) {
                    const uint32_t s = exponent_of(run[i]);
                    acc |= static_cast<uint64_t>(rev[s]) << fill;
                    fill += lens[s];
                    bits_j += lens[s];
                    if (fill >= 32) {
                        const uint32_t out = static_cast<uint32_t>(acc);
                        std::memcpy(area + 4 * word, &out, 4);
                        ++word;
                        acc >>= 32;
                        fill -= 32;
                    }
                }
            }
            const uint16_t sb = static_cast<uint16_t>(bits_j);
            std::memcpy(blk + 8 + 2 * j, &sb, 2);
        }
        if (fill) {
            const uint32_t out = static_cast<uint32_t>(acc);
            std::memcpy(area + 4 * word, &out, 4);
        }
    }
}

}  // namespace fluxmoe
