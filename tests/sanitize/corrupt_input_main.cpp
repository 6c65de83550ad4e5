// Host-side sanitizer run: the oracle's decoders and the library's CPU sources (model validation / load, fit)
// on arbitrary bytes, in exactly-sized heap buffers, built with -fsanitize=address,undefined.  Any read or
// write outside a buffer, any shift or index out of range, ends the program with a report and a non-zero
// status.  Built and run by tests/test_sanitizers.py; no GPU code, no HIP call is made.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ecco.h"
#include "ecco_paper_block.h"
#include "../../oracle/ecco_oracle.h"
#include "../../oracle/ecco_paper_block.h"

// the model source asks the kernel source for a device address when a model is uploaded; this program has no kernel
// source and uploads nothing
namespace ecco {
int init_device_scratch(int) { return 0; }
}  // namespace ecco

namespace {

struct Rng {
    uint64_t s;
    uint64_t next() {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
};

#define REQUIRE(cond) do { if (!(cond)) { std::fprintf(stderr, "requirement failed at line %d: %s\n", __LINE__, #cond); std::exit(2); } } while (0)

// a valid model with S patterns: ascending centroids, and per pattern the optimal code lengths (at most 12 bits) of a
// random histogram, some flat and some steep, so that short and long codes both occur
void make_model(int S, Rng& rng, std::vector<uint16_t>& cent, std::vector<uint8_t>& lens) {
    cent.assign((size_t)S * 16, 0);
    lens.assign((size_t)S * 16, 4);
    for (int p = 0; p < S; ++p) {
        for (int k = 0; k < 16; ++k) {
            const float v = -1.0f + 2.0f * (float)k / 15.0f;
            cent[(size_t)p * 16 + k] = oracle_f2h(v * (0.5f + 0.5f * (float)((p % 7) + 1) / 7.0f));
        }
        uint64_t counts[16];
        const int steep = (int)(rng.next() % 4);  // 0: flat ... 3: counts spread over 45 octaves
        for (int k = 0; k < 16; ++k) counts[k] = 1 + (rng.next() % 1000) * (steep ? (1ull << ((rng.next() % 16) * steep)) : 1ull);
        REQUIRE(oracle_limited_lengths(counts, 16, 12, &lens[(size_t)p * 16]) == 0);
    }
}

void oracle_on_junk(Rng& rng) {
    for (int S : {1, 3, 16, 64}) {
        std::vector<uint16_t> cent;
        std::vector<uint8_t> lens;
        make_model(S, rng, cent, lens);
        // pattern 0 gets codes of every length up to 12 bits
        uint64_t counts[16];
        for (int k = 0; k < 16; ++k) counts[k] = 1ull << (2 * (15 - k));
        REQUIRE(oracle_limited_lengths(counts, 16, 12, &lens[0]) == 0);
        REQUIRE(oracle_verify_model(cent.data(), lens.data(), S) == 0);
        const size_t n = 257;
        std::vector<uint8_t> blocks(n * 64);
        std::vector<uint32_t> meta(n);
        for (auto& b : blocks) b = (uint8_t)rng.next();
        for (auto& m : meta) m = (uint32_t)rng.next() & 0xFFFF7BFFu;  // finite scale; pattern id, raw flag and start position arbitrary
        for (size_t g = 0; g < 8; ++g) std::memset(&blocks[g * 64], g & 1 ? 0xFF : 0x00, 64);  // all ones: the longest codes; all zeros: the shortest
        std::vector<uint8_t> idx(n * 128);
        std::vector<uint16_t> used(n), dst(n * 128);
        oracle_decode_indices(lens.data(), S, blocks.data(), meta.data(), n, idx.data(), used.data());
        for (uint8_t v : idx) REQUIRE(v < 16);
        oracle_decode(cent.data(), lens.data(), S, blocks.data(), meta.data(), n, dst.data());
        // every block once more on its own, in a heap buffer of exactly 64 bytes: inside an array a read past a
        // block's end lands in the next block and goes unnoticed
        for (size_t g = 0; g < n; ++g) {
            std::vector<uint8_t> one(blocks.begin() + (long)(g * 64), blocks.begin() + (long)(g * 64 + 64));
            std::vector<uint8_t> one_idx(128);
            std::vector<uint16_t> one_dst(128);
            uint16_t one_used = 0;
            oracle_decode_indices(lens.data(), S, one.data(), &meta[g], 1, one_idx.data(), &one_used);
            REQUIRE(std::memcmp(one_idx.data(), &idx[g * 128], 128) == 0);
            oracle_decode(cent.data(), lens.data(), S, one.data(), &meta[g], 1, one_dst.data());
            REQUIRE(std::memcmp(one_dst.data(), &dst[g * 128], 256) == 0);
        }
        // consumers over the same junk: a 1 x (257 x 128) matrix, and a cache of 257 tokens
        std::vector<uint16_t> x(n * 128);
        for (auto& v : x) v = (uint16_t)(rng.next() & 0x3FFF);
        std::vector<double> y(1);
        oracle_gemv(cent.data(), lens.data(), S, blocks.data(), meta.data(), 1, (int)(n * 128), x.data(), 1, y.data());
        const int32_t seq = (int32_t)n;
        std::vector<double> out(128);
        oracle_kv_attend(cent.data(), lens.data(), S, cent.data(), lens.data(), S, x.data(), blocks.data(), meta.data(),
                         blocks.data(), meta.data(), &seq, 1, 1, (int)n, out.data());
        // and the encoder on extreme finite values
        std::vector<uint16_t> src(6 * 128);
        for (size_t i = 0; i < src.size(); ++i) {
            const size_t g = i / 128;
            src[i] = g == 0 ? 0 : g == 1 ? 0x7BFF : g == 2 ? 0xFBFF : g == 3 ? 0x0001 : g == 4 ? (uint16_t)(0x8000 | (i & 0x3FF)) : (uint16_t)(rng.next() & 0x7BFF);
        }
        std::vector<uint8_t> eb(6 * 64);
        std::vector<uint32_t> em(6);
        oracle_encode(cent.data(), lens.data(), S, src.data(), 6, eb.data(), em.data());
        oracle_encode_minmax(cent.data(), lens.data(), S, src.data(), 6, eb.data(), em.data());
    }
    // the activation codec on junk
    {
        const size_t n = 100;
        std::vector<uint8_t> blocks(n * 64);
        for (auto& b : blocks) b = (uint8_t)rng.next();
        std::vector<uint16_t> dst(n * 64);
        oracle_act_decode(blocks.data(), n, dst.data());
        for (auto& v : dst) v &= 0x7BFF;
        oracle_act_encode(dst.data(), n, blocks.data());
    }
}

void paper_block_oracle_on_junk(Rng& rng) {
    for (int S : {1, 5, 64}) {
        std::vector<uint16_t> cent((size_t)S * 15);
        std::vector<uint8_t> lens((size_t)S * 4 * 16), kp((size_t)S);
        for (int p = 0; p < S; ++p)
            for (int k = 0; k < 15; ++k) cent[(size_t)p * 15 + k] = oracle_f2h((-1.0f + 2.0f * (float)k / 14.0f) * (0.3f + 0.7f * (float)(p % 5) / 4.0f));
        static const uint8_t books[2][16] = {{4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4, 4}, {2, 2, 3, 4, 5, 6, 7, 8, 8, 4, 5, 6, 7, 8, 8, 3}};
        for (int p = 0; p < S; ++p)
            for (int h = 0; h < 4; ++h) {
                const uint8_t* b = books[(p + h) & 1];
                uint32_t kraft = 0;
                for (int k = 0; k < 16; ++k) kraft += 1u << (8 - b[k]);
                std::memcpy(&lens[((size_t)p * 4 + h) * 16], kraft == 256u ? b : books[0], 16);
            }
        // pattern-id code lengths: a complete code over S symbols
        if (S == 1) kp[0] = 1;
        else if (S == 5) { const uint8_t l[5] = {1, 2, 3, 4, 4}; std::memcpy(kp.data(), l, 5); }
        else for (int p = 0; p < S; ++p) kp[(size_t)p] = 6;
        pb_model m{S, -6, cent.data(), lens.data(), kp.data()};
        REQUIRE(pb_verify_model(&m) == 0);
        const size_t n = 200;
        std::vector<uint8_t> blocks(n * 64), coded(n), outl(n);
        for (auto& b : blocks) b = (uint8_t)rng.next();
        for (size_t g = 0; g < 6; ++g) std::memset(&blocks[g * 64], g & 1 ? 0xFF : 0x00, 64);
        std::vector<uint16_t> dst(n * 128);
        pb_decode(&m, blocks.data(), n, dst.data(), coded.data(), outl.data());
        for (size_t g = 0; g < n; ++g) {  // and each block alone in a buffer of exactly 64 bytes
            std::vector<uint8_t> one(blocks.begin() + (long)(g * 64), blocks.begin() + (long)(g * 64 + 64));
            std::vector<uint16_t> one_dst(128);
            pb_decode(&m, one.data(), 1, one_dst.data(), nullptr, nullptr);
            REQUIRE(std::memcmp(one_dst.data(), &dst[g * 128], 256) == 0);
        }
        std::vector<uint16_t> x(n * 128);
        for (auto& v : x) v = (uint16_t)(rng.next() & 0x3FFF);
        double y = 0.0;
        pb_gemv(&m, blocks.data(), 1, (int)(n * 128), x.data(), &y);
        for (auto& v : x) v = (uint16_t)((rng.next() & 0xFFFF) % 0x7C00u);  // finite
        pb_encode(&m, x.data(), n, blocks.data());
    }
}

void library_host_code_on_junk(Rng& rng) {
    // serialised models: arbitrary bytes, truncated and bit-flipped copies of a valid blob must be refused or accepted
    // without touching memory outside the buffer
    std::vector<uint16_t> cent;
    std::vector<uint8_t> lens;
    make_model(16, rng, cent, lens);
    ecco_model* m = nullptr;
    REQUIRE(ecco_model_create(cent.data(), lens.data(), 16, &m) == ECCO_OK);
    size_t need = 0;
    REQUIRE(ecco_model_save(m, nullptr, 0, &need) == ECCO_OK);
    std::vector<uint8_t> blob(need);
    REQUIRE(ecco_model_save(m, blob.data(), blob.size(), &need) == ECCO_OK);
    ecco_model_free(m);
    for (size_t len = 0; len <= blob.size(); len += (len < 40 ? 1 : 37)) {
        std::vector<uint8_t> cut(blob.begin(), blob.begin() + (long)len);  // exactly-sized copy
        ecco_model* t = nullptr;
        const int rc = ecco_model_load(cut.data(), cut.size(), &t);
        if (rc == ECCO_OK) ecco_model_free(t);
    }
    for (int trial = 0; trial < 400; ++trial) {
        std::vector<uint8_t> b(blob);
        const int flips = 1 + (int)(rng.next() % 4);
        for (int f = 0; f < flips; ++f) b[rng.next() % b.size()] ^= (uint8_t)(1u << (rng.next() % 8));
        ecco_model* t = nullptr;
        if (ecco_model_load(b.data(), b.size(), &t) == ECCO_OK) ecco_model_free(t);
        std::vector<uint8_t> junk(rng.next() % 3000);
        for (auto& v : junk) v = (uint8_t)rng.next();
        if (ecco_model_load(junk.data(), junk.size(), &t) == ECCO_OK) ecco_model_free(t);
    }
    // the CPU fit on small inputs, edge values included
    for (int S : {1, 2, 16}) {
        std::vector<uint16_t> data(40 * 128);
        for (size_t i = 0; i < data.size(); ++i) data[i] = (uint16_t)((rng.next() & 0xFFFF) % 0x7C00u) | (uint16_t)((rng.next() & 1) << 15);
        std::memset(data.data(), 0, 256);  // an all-zero group
        ecco_model* t = nullptr;
        REQUIRE(ecco_fit_patterns(data.data(), data.size(), S, 12, 7, &t) == ECCO_OK);
        ecco_model_free(t);
        REQUIRE(ecco_fit_patterns(data.data(), 128, S, 4, 7, &t) == ECCO_OK);
        ecco_model_free(t);
    }
    // the self-contained block's model: same treatment
    {
        std::vector<uint16_t> data(64 * 128);
        for (auto& v : data) v = (uint16_t)((rng.next() & 0xFFFF) % 0x7C00u) | (uint16_t)((rng.next() & 1) << 15);
        ecco_pb_model* pm = nullptr;
        REQUIRE(ecco_pb_fit(data.data(), data.size(), 4, 3, &pm) == ECCO_OK);
        size_t w = 0;
        REQUIRE(ecco_pb_model_save(pm, nullptr, 0, &w) == ECCO_OK);
        std::vector<uint8_t> pblob(w);
        REQUIRE(ecco_pb_model_save(pm, pblob.data(), pblob.size(), &w) == ECCO_OK);
        ecco_pb_model_free(pm);
        for (size_t len = 0; len <= pblob.size(); len += (len < 40 ? 1 : 29)) {
            std::vector<uint8_t> cut(pblob.begin(), pblob.begin() + (long)len);
            ecco_pb_model* t = nullptr;
            if (ecco_pb_model_load(cut.data(), cut.size(), &t) == ECCO_OK) ecco_pb_model_free(t);
        }
        for (int trial = 0; trial < 300; ++trial) {
            std::vector<uint8_t> b(pblob);
            b[rng.next() % b.size()] ^= (uint8_t)(1u << (rng.next() % 8));
            ecco_pb_model* t = nullptr;
            if (ecco_pb_model_load(b.data(), b.size(), &t) == ECCO_OK) ecco_pb_model_free(t);
        }
    }
}

}  // namespace

int main() {
    Rng rng{2025};
    oracle_set_threads(1);
    oracle_on_junk(rng);
    std::puts("oracle decoders, consumers and encoder on arbitrary bytes: clean");
    paper_block_oracle_on_junk(rng);
    std::puts("self-contained block oracle on arbitrary bytes: clean");
    library_host_code_on_junk(rng);
    std::puts("library host code (model load / create / fit) on arbitrary bytes: clean");
    return 0;
}
