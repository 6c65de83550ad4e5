// Internal definitions of libecco: the model object and the layout of its device tables.
#pragma once

#include <cstddef>
#include <cstdint>

#include "ecco.h"

namespace ecco {

constexpr int kGroup = ECCO_GROUP;
constexpr int kK = ECCO_K;
constexpr int kMaxLen = ECCO_MAX_LEN;
constexpr int kMaxS = ECCO_MAX_S;
constexpr int kBlockWords = ECCO_BLOCK_BYTES / 4;

// Short-code table: a peek of kPeekBits stream bits (first bit in bit 0) selects one byte,
// (code length << 4) | index; 0 marks a code longer than kPeekBits.  Slot kMaxS is the raw-mode
// table (length 4, index = low nibble of the peek), so raw blocks take the same code path.
constexpr int kPeekBits = 8;
constexpr int kLutSlots = kMaxS + 1;
constexpr int kRawSlot = kMaxS;

// Pair table for the fused kernels: a peek of kPairBits stream bits selects a 16-bit entry
//   bits 3:0  first index, bits 7:4 second index (0 when absent),
//   bits 11:8 stream bits consumed, bits 13:12 number of indices decoded (1 or 2), 0 = long code.
constexpr int kPairBits = 10;

// Device tables, one allocation; offsets in bytes.
struct DevLayout {
    static constexpr size_t cent = 0;                                      // half  [kMaxS][16]
    static constexpr size_t lut8 = cent + kMaxS * kK * 2;                  // u8    [kLutSlots][256]
    static constexpr size_t longtab = lut8 + kLutSlots * 256;              // u32   [kMaxS][16]
    static constexpr size_t enc = longtab + kMaxS * kK * 4;                // u32   [kMaxS][16]
    static constexpr size_t pair = enc + kMaxS * kK * 4;                   // u16   [kLutSlots][1 << kPairBits]
    static constexpr size_t total = pair + (size_t)kLutSlots * (1u << kPairBits) * 2;
};

// longtab entry j (canonical position j): bits 11:0 the code left-aligned in 12 bits,
// bits 15:12 the index, bits 20:16 the code length.
// enc entry k: bits 15:0 the code with its bits reversed (first code bit in bit 0), bits 20:16 length.

}  // namespace ecco

struct ecco_model {
    int S = 0;
    uint16_t cent[ecco::kMaxS * ecco::kK] = {};
    uint8_t lens[ecco::kMaxS * ecco::kK] = {};
    uint16_t codes[ecco::kMaxS * ecco::kK] = {};  // canonical codes, derived from lens
    int device = -1;
    unsigned char* dev = nullptr;  // DevLayout::total bytes on `device`
};

namespace ecco {

// validation shared by create / load; returns ECCO_OK or ECCO_EFORMAT
int validate_tables(const uint16_t* cent, const uint8_t* lens, int S);
void derive_codes(ecco_model* m);
// fills a host image of the device tables (DevLayout::total bytes)
void build_device_image(const ecco_model* m, unsigned char* img);

// host-side half conversion helpers (compiler-provided _Float16 arithmetic)
inline float half_bits_to_float(uint16_t h) {
    _Float16 v;
    __builtin_memcpy(&v, &h, 2);
    return (float)v;
}
inline uint16_t float_to_half_bits(float f) {
    _Float16 v = (_Float16)f;
    uint16_t h;
    __builtin_memcpy(&h, &v, 2);
    return h;
}

}  // namespace ecco
