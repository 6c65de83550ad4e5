// Internal definitions of the self-contained block format (include/ecco_paper_block.h): the model object and
// the layout of its device tables.
#pragma once

#include <cstddef>
#include <cstdint>

#include "ecco_paper_block.h"

namespace ecco_pb {

constexpr int kGroup = ECCO_GROUP;
constexpr int kCent = ECCO_PB_CENTROIDS;   // centroids per pattern
constexpr int kSym = 16;                   // indices: 15 centroids + the element of largest magnitude
constexpr int kBooks = ECCO_PB_BOOKS;
constexpr int kMinLen = ECCO_PB_MIN_LEN;
constexpr int kMaxLen = ECCO_PB_MAX_LEN;
constexpr int kMaxS = ECCO_MAX_S;
constexpr int kBlockWords = ECCO_BLOCK_BYTES / 4;
constexpr int kBlockBits = ECCO_BLOCK_BYTES * 8;
constexpr int kOutlierBits = 15;

// Device memory of a model, one allocation, in 32-bit words:
//   lut     [S * 4][256] bytes   8-bit peek -> (index << 4) | code length, one table per (pattern, codebook)
//   kplut   [256] 16-bit         8-bit peek -> (pattern << 8) | code length of the pattern id; no match: (S - 1, 8)
//   cent    [S][16] FP16         centroids; entry 15 = 1.0 (index 15 stands for the scale itself)
//   fp8     [256] FP16           value of every 8-bit float times 2^texp
//   enc     [S * 4][16]          code | length << 16 per index
//   kpenc   [S] (padded to 4)    code | length << 16 per pattern id
// The first four are what the decoder stages in LDS, the last four what the encoder stages.
struct DevLayout {
    int S;
    constexpr size_t lut() const { return 0; }
    constexpr size_t kplut() const { return (size_t)S * kBooks * 64; }
    constexpr size_t cent() const { return kplut() + 128; }
    constexpr size_t fp8() const { return cent() + (size_t)S * 8; }
    constexpr size_t enc() const { return fp8() + 128; }
    constexpr size_t kpenc() const { return enc() + (size_t)S * kBooks * kSym; }
    constexpr size_t total_words() const { return kpenc() + (((size_t)S + 3) & ~(size_t)3); }
    constexpr size_t decode_words() const { return enc(); }            // lut .. fp8
    constexpr size_t encode_words() const { return total_words() - cent(); }  // cent .. kpenc
};

// the 8-bit float of the format
inline double fp8_value(uint8_t b) {
    const int e = (b >> 3) & 15, mant = b & 7;
    double mag = e == 0 ? (double)mant / 512.0 : (double)(8 + mant) * (e >= 10 ? (double)(1 << (e - 10)) : 1.0 / (double)(1 << (10 - e)));
    return (b & 0x80) ? -mag : mag;
}

}  // namespace ecco_pb

struct ecco_pb_model {
    int S = 0;
    int texp = 0;
    uint16_t cent[ecco_pb::kMaxS * ecco_pb::kCent] = {};
    uint8_t lens[ecco_pb::kMaxS * ecco_pb::kBooks * ecco_pb::kSym] = {};
    uint8_t kp_lens[ecco_pb::kMaxS] = {};
    uint16_t codes[ecco_pb::kMaxS * ecco_pb::kBooks * ecco_pb::kSym] = {};
    uint16_t kp_codes[ecco_pb::kMaxS] = {};
    int device = -1;
    uint32_t* dev = nullptr;
};
