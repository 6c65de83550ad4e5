// CPU oracle for the paper's self-contained 4x block -- TEST INFRASTRUCTURE ONLY (see ecco_paper_block.h).
//
// What the paper fixes (Section 3.2; Sections 4.2 and 4.3 for the 4x units): groups of 128 values; the group's
// absolute maximum, divided by a per-tensor power-of-two scale and stored as FP8, is the group scale; 15
// centroids per shared pattern for the other 127 values and index 15 for the absolute maximum itself; H = 4
// Huffman codebooks per pattern, the one giving the shortest total length is chosen (2-bit ID_HF); the pattern
// id (ID_KP) is Huffman coded; code lengths are 2..8 bits; a block that overflows is clipped; a block with
// spare room is padded with the largest remaining magnitudes, 15 bits each (7-bit position, FP8 value on the
// per-tensor scale), which replace the centroid values at their positions when decoding.
// This build's reading of what the paper leaves open (its figure of the block is not available):
//   * FP8 = 1-4-3 bits, bias 7, subnormals, every bit pattern a finite number (largest 480); round to nearest,
//     ties to even, saturating.  The sign bit of the scale byte is the sign of the absolute-maximum element, so
//     index 15 reconstructs to the signed scale.
//   * bit stream as in the other format: 16 little-endian 32-bit words, most significant bit of each first.
//     Order of fields: scale byte, ID_HF (2 bits), ID_KP code, the 128 data codes, outlier entries (position,
//     then value), zero fill.  Every field is written most significant bit first.
//   * clipping is literal truncation of the stream at bit 512.  A value is present iff its whole code lies inside
//     the block; because the codes are prefix-free the decoder can tell (the code it reads at the cut always
//     ends beyond bit 512).  Values that are not present decode to +0.
//   * outliers follow only if all 128 values are present; their number is floor(spare bits / 15) (at most 16);
//     candidates are all elements but the absolute maximum, by decreasing magnitude, lower position first on ties.
//   * values are compared with the reconstructed centroids fp16(c * |scale|) as in the other format (nearest,
//     lowest index on ties; squared errors summed in the balanced fp32 tree with the absolute-maximum element
//     contributing 0; lowest pattern and lowest codebook on ties).
//   * an unmatched pattern-id code (only possible in a block the encoder did not write) selects pattern S - 1
//     and consumes 8 bits.
// Parity status: FP8 conversion, block layout, clipping and outlier rules are pinned in tests/test_paper_block_pins.py
// (exact rationals, hand-packed blocks, brute force); fitted models: invariants only (parity unpinned, as for the
// other format).
#include "ecco_paper_block.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "ecco_oracle.h"

namespace {

constexpr int G = PB_GROUP;
constexpr int KC = PB_CENTROIDS;
constexpr int NSYM = PB_SYMBOLS;

int stream_bit(const uint8_t* blk, int j) {  // bits at and past 512 read as 0
    if (j >= 8 * PB_BLOCK_BYTES) return 0;
    int word = j >> 5, bit = 31 - (j & 31);
    return (blk[4 * word + (bit >> 3)] >> (bit & 7)) & 1;
}

void set_stream_bit(uint8_t* blk, int j, int b) {
    if (j >= 8 * PB_BLOCK_BYTES || !b) return;  // literal truncation: what lies beyond the block is dropped
    int word = j >> 5, bit = 31 - (j & 31);
    blk[4 * word + (bit >> 3)] |= (uint8_t)(1u << (bit & 7));
}

void put_field(uint8_t* blk, int* pos, uint32_t value, int nbits) {  // most significant bit first
    for (int b = nbits - 1; b >= 0; --b) set_stream_bit(blk, (*pos)++, (value >> b) & 1);
}

uint32_t get_field(const uint8_t* blk, int pos, int nbits) {
    uint32_t v = 0;
    for (int b = 0; b < nbits; ++b) v = (v << 1) | (uint32_t)stream_bit(blk, pos + b);
    return v;
}

// fp16 bit pattern of fp8 value times 2^texp: exact for texp in -15..7 (4 significant bits, within the fp16 range)
uint16_t fp8_scaled_half(uint8_t b, int texp) {
    return oracle_f2h((float)std::ldexp(pb_fp8_value(b), texp));
}

struct Books {
    std::vector<uint16_t> codes;     // [S][4][16]
    std::vector<uint16_t> kp_codes;  // [S]
};

Books derive_codes(const pb_model* m) {
    Books b;
    b.codes.resize((size_t)m->S * PB_BOOKS * NSYM);
    for (int t = 0; t < m->S * PB_BOOKS; ++t) oracle_canonical_codes(m->lens + t * NSYM, NSYM, b.codes.data() + t * NSYM);
    b.kp_codes.resize((size_t)m->S);
    oracle_canonical_codes(m->kp_lens, m->S, b.kp_codes.data());
    return b;
}

}  // namespace

double pb_fp8_value(uint8_t b) {
    int e = (b >> 3) & 15, mant = b & 7;
    double mag = e == 0 ? std::ldexp((double)mant, -9) : std::ldexp((double)(8 + mant), e - 10);
    return (b & 0x80) ? -mag : mag;
}

uint8_t pb_fp8_round(double v) {
    uint8_t sign = std::signbit(v) ? 0x80 : 0;
    double a = std::fabs(v);
    // the non-negative values in increasing order are exactly the codes 0..127: pick the nearest, the even code on a tie
    int lo = 0, hi = 127;
    if (a >= pb_fp8_value(127)) return (uint8_t)(sign | 127);
    while (hi - lo > 1) {  // invariant: value(lo) <= a < value(hi)
        int mid = (lo + hi) / 2;
        if (pb_fp8_value((uint8_t)mid) <= a) lo = mid; else hi = mid;
    }
    double dl = a - pb_fp8_value((uint8_t)lo), dh = pb_fp8_value((uint8_t)hi) - a;
    int pick = dl < dh ? lo : dh < dl ? hi : ((lo & 1) ? hi : lo);
    return (uint8_t)(sign | pick);
}

int pb_verify_model(const pb_model* m) {
    if (m->S < 1 || m->S > PB_MAX_S) return 1;
    if (m->texp < -15 || m->texp > 7) return 2;
    for (int p = 0; p < m->S; ++p) {
        for (int k = 0; k < KC; ++k) {
            uint16_t h = m->cent[p * KC + k];
            if ((h & 0x7C00) == 0x7C00) return 3;
            float v = oracle_h2f(h);
            if (v < -1.0f || v > 1.0f) return 4;
            if (k && v < oracle_h2f(m->cent[p * KC + k - 1])) return 5;
        }
        for (int h = 0; h < PB_BOOKS; ++h) {
            const uint8_t* l = m->lens + (p * PB_BOOKS + h) * NSYM;
            long kraft = 0;
            for (int k = 0; k < NSYM; ++k) {
                if (l[k] < PB_MIN_LEN || l[k] > PB_MAX_LEN) return 6;
                kraft += 1L << (PB_MAX_LEN - l[k]);
            }
            if (kraft != (1L << PB_MAX_LEN)) return 7;
        }
    }
    long kraft = 0;
    for (int p = 0; p < m->S; ++p) {
        if (m->kp_lens[p] < 1 || m->kp_lens[p] > 8) return 8;
        kraft += 1L << (8 - m->kp_lens[p]);
    }
    if (kraft > 256 || (m->S >= 2 && kraft != 256)) return 9;
    return 0;
}

void pb_quantize_group(const pb_model* m, const uint16_t* x, int* amax_pos, uint8_t* scale8, int* pattern, int* book,
                       uint8_t* idx) {
    // the absolute maximum (first position on ties) and its FP8 image on the tensor scale
    int a = 0;
    for (int i = 1; i < G; ++i)
        if ((x[i] & 0x7FFF) > (x[a] & 0x7FFF)) a = i;
    uint8_t s8 = pb_fp8_round(std::ldexp((double)oracle_h2f(x[a]), -m->texp));
    uint16_t sabs = (uint16_t)(fp8_scaled_half(s8, m->texp) & 0x7FFF);
    int best_p = 0;
    float best_sse = 0.0f;
    uint8_t best_idx[G];
    for (int p = 0; p < m->S; ++p) {
        float r[KC];
        for (int k = 0; k < KC; ++k) r[k] = oracle_h2f(oracle_dequant(m->cent[p * KC + k], sabs));
        float e[G];
        uint8_t id[G];
        for (int i = 0; i < G; ++i) {
            if (i == a) { e[i] = 0.0f; id[i] = 15; continue; }
            float xi = oracle_h2f(x[i]);
            int bk = 0;
            float bd = std::fabs(xi - r[0]);
            for (int k = 1; k < KC; ++k) {
                float d = std::fabs(xi - r[k]);
                if (d < bd) { bd = d; bk = k; }
            }
            float d = xi - r[bk];
            e[i] = d * d;
            id[i] = (uint8_t)bk;
        }
        for (int stride = 1; stride < G; stride <<= 1)
            for (int i = 0; i < G; i += 2 * stride) e[i] = e[i] + e[i + stride];
        if (p == 0 || e[0] < best_sse) { best_sse = e[0]; best_p = p; std::memcpy(best_idx, id, G); }
    }
    // the codebook with the shortest total length
    int best_h = 0, best_total = 0;
    for (int h = 0; h < PB_BOOKS; ++h) {
        const uint8_t* l = m->lens + (best_p * PB_BOOKS + h) * NSYM;
        int total = 0;
        for (int i = 0; i < G; ++i) total += l[best_idx[i]];
        if (h == 0 || total < best_total) { best_total = total; best_h = h; }
    }
    *amax_pos = a; *scale8 = s8; *pattern = best_p; *book = best_h;
    std::memcpy(idx, best_idx, G);
}

void pb_encode(const pb_model* m, const uint16_t* src, size_t n_groups, uint8_t* blocks) {
    Books bk = derive_codes(m);
    for (size_t g = 0; g < n_groups; ++g) {
        const uint16_t* x = src + g * G;
        uint8_t* blk = blocks + g * PB_BLOCK_BYTES;
        std::memset(blk, 0, PB_BLOCK_BYTES);
        int a, p, h;
        uint8_t s8, idx[G];
        pb_quantize_group(m, x, &a, &s8, &p, &h, idx);
        int pos = 0;
        put_field(blk, &pos, s8, 8);
        put_field(blk, &pos, (uint32_t)h, 2);
        put_field(blk, &pos, bk.kp_codes[p], m->kp_lens[p]);
        const uint8_t* l = m->lens + (p * PB_BOOKS + h) * NSYM;
        const uint16_t* c = bk.codes.data() + (p * PB_BOOKS + h) * NSYM;
        for (int i = 0; i < G; ++i) put_field(blk, &pos, c[idx[i]], l[idx[i]]);  // bits past 512 are dropped
        if (pos > 8 * PB_BLOCK_BYTES) continue;                                   // clipped: no room for outliers
        int slots = (8 * PB_BLOCK_BYTES - pos) / PB_OUTLIER_BITS;
        std::vector<int> order;
        for (int i = 0; i < G; ++i) if (i != a) order.push_back(i);
        std::stable_sort(order.begin(), order.end(), [&](int i, int j) { return (x[i] & 0x7FFF) > (x[j] & 0x7FFF); });
        for (int j = 0; j < slots && j < (int)order.size(); ++j) {
            int i = order[j];
            put_field(blk, &pos, (uint32_t)i, 7);
            put_field(blk, &pos, pb_fp8_round(std::ldexp((double)oracle_h2f(x[i]), -m->texp)), 8);
        }
    }
}

void pb_decode(const pb_model* m, const uint8_t* blocks, size_t n_groups, uint16_t* dst, uint8_t* n_coded_out, uint8_t* n_out_out) {
    Books bk = derive_codes(m);
    for (size_t g = 0; g < n_groups; ++g) {
        const uint8_t* blk = blocks + g * PB_BLOCK_BYTES;
        uint16_t* out = dst + g * G;
        uint8_t s8 = (uint8_t)get_field(blk, 0, 8);
        uint16_t sv = fp8_scaled_half(s8, m->texp), sabs = (uint16_t)(sv & 0x7FFF);
        int h = (int)get_field(blk, 8, 2);
        // pattern id: read bits until they equal one of the pattern-id codes
        int p = m->S - 1, pos = 10 + 8;
        {
            uint32_t code = 0;
            bool found = false;
            for (int len = 1; len <= 8 && !found; ++len) {
                code = (code << 1) | (uint32_t)stream_bit(blk, 10 + len - 1);
                for (int q = 0; q < m->S; ++q)
                    if (m->kp_lens[q] == len && bk.kp_codes[q] == code) { p = q; pos = 10 + len; found = true; break; }
            }
        }
        const uint8_t* l = m->lens + (p * PB_BOOKS + h) * NSYM;
        const uint16_t* c = bk.codes.data() + (p * PB_BOOKS + h) * NSYM;
        int n_coded = 0;
        for (int i = 0; i < G; ++i) out[i] = 0;
        for (int i = 0; i < G; ++i) {
            uint32_t code = 0;
            int len = 0, sym = -1;
            while (sym < 0 && len < PB_MAX_LEN) {
                code = (code << 1) | (uint32_t)stream_bit(blk, pos + len);
                ++len;
                for (int k = 0; k < NSYM; ++k)
                    if (l[k] == len && c[k] == code) sym = k;
            }
            // a complete code (Kraft sum 1) always matches within 8 bits
            if (sym < 0 || pos + len > 8 * PB_BLOCK_BYTES) break;  // the code ends beyond the block: this and all later values are absent
            out[i] = sym == 15 ? sv : oracle_dequant(m->cent[p * KC + sym], sabs);
            pos += len;
            ++n_coded;
        }
        int n_out = 0;
        if (n_coded == G) {
            n_out = (8 * PB_BLOCK_BYTES - pos) / PB_OUTLIER_BITS;
            for (int j = 0; j < n_out; ++j) {
                int where = (int)get_field(blk, pos, 7);
                uint8_t v8 = (uint8_t)get_field(blk, pos + 7, 8);
                out[where] = fp8_scaled_half(v8, m->texp);
                pos += PB_OUTLIER_BITS;
            }
        }
        if (n_coded_out) n_coded_out[g] = (uint8_t)n_coded;
        if (n_out_out) n_out_out[g] = (uint8_t)n_out;
    }
}

// the consumer of the decompressed weights (Section 2.1: decode-phase projections are matrix-vector products)
void pb_gemv(const pb_model* m, const uint8_t* blocks, int rows, int cols, const uint16_t* x, double* y) {
    const int gpr = cols / G;
    std::vector<uint16_t> w((size_t)cols);
    for (int r = 0; r < rows; ++r) {
        pb_decode(m, blocks + (size_t)r * gpr * PB_BLOCK_BYTES, (size_t)gpr, w.data(), nullptr, nullptr);
        double acc = 0.0;
        for (int c = 0; c < cols; ++c) acc += (double)oracle_h2f(w[(size_t)c]) * (double)oracle_h2f(x[c]);
        y[r] = acc;
    }
}
