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

// Decode table: a peek at the next kPeekBits stream bits (first bit most significant) selects one
// 32-bit entry per pattern:
//   bits 31:16  the centroid (FP16 bits) of the index whose code starts the peek
//   bits 11:8   that index
//   bits  7:0   the code length; 0 marks a code longer than kPeekBits (resolved through `longtab`)
// Raw-mode blocks use a 16-entry table per pattern, indexed by the next 4 bits, of the same entry
// format (length 4), so raw and Huffman blocks run the same instructions with a different shift.
constexpr int kPeekBits = 8;
constexpr int kPeekEntries = 1 << kPeekBits;

// Device memory of a model, one allocation, in 32-bit words:
//   compact tables  [enc S x 16][centroids S x 8][longtab S x 16]   (a few KB; kernels expand them in LDS)
// The decode table itself (S x 256 entries) is never stored in global memory: every workgroup
// builds it in LDS from `enc` and the centroids, which costs less than fetching 64 KB per workgroup.
struct DevLayout {
    int S;
    constexpr size_t enc() const { return 0; }
    constexpr size_t cent() const { return (size_t)S * kK; }
    constexpr size_t longtab() const { return cent() + (size_t)S * kK / 2; }
    constexpr size_t table_words() const { return longtab() + (size_t)S * kK; }
    constexpr size_t image_words() const { return table_words(); }
    constexpr size_t total_bytes() const { return image_words() * 4; }
};

// longtab entry j (canonical position j): bits 11:0 the code left-aligned in 12 bits,
// bits 15:12 the index, bits 20:16 the code length.
// enc entry k: bits 15:0 the code (first code bit most significant), bits 20:16 its length.

}  // namespace ecco

struct ecco_model {
    int S = 0;
    uint16_t cent[ecco::kMaxS * ecco::kK] = {};
    uint8_t lens[ecco::kMaxS * ecco::kK] = {};
    uint16_t codes[ecco::kMaxS * ecco::kK] = {};  // canonical codes, derived from lens
    int device = -1;
    int max_len = 0;               // longest code length in the model
    uint32_t* dev = nullptr;       // DevLayout{S}.total_bytes() on `device`
};

namespace ecco {

// validation shared by create / load; returns ECCO_OK or ECCO_EFORMAT
int validate_tables(const uint16_t* cent, const uint8_t* lens, int S);
void derive_codes(ecco_model* m);
// fills a host image of the device tables (DevLayout{S}.image_words() words; counters zero)
void build_device_image(const ecco_model* m, uint32_t* img);

// looks up, for `device` (which must be current), the device address of the static scratch array that
// ecco_kv_attend_gqa_noalloc uses; defined beside that array in ecco_kernels.hip.  ECCO_OK or ECCO_EHIP.
int init_device_scratch(int device);

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
