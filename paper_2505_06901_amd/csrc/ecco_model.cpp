// The model object: validation, canonical code derivation, the decode / encode tables, the
// serialised form, and the one-time upload (Section 4.2: shared patterns and codebooks are
// tensor-level metadata, loaded once before any compressed block is read).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "ecco_internal.h"

namespace ecco {

int validate_tables(const uint16_t* cent, const uint8_t* lens, int S) {
    if (S < 1 || S > kMaxS) return ECCO_EFORMAT;
    for (int p = 0; p < S; ++p) {
        uint32_t kraft = 0;
        for (int k = 0; k < kK; ++k) {
            uint16_t c = cent[p * kK + k];
            if ((c & 0x7C00) == 0x7C00) return ECCO_EFORMAT;          // Inf / NaN
            if ((c & 0x7FFF) > 0x3C00) return ECCO_EFORMAT;           // |c| > 1
            if (k && half_bits_to_float(c) < half_bits_to_float(cent[p * kK + k - 1])) return ECCO_EFORMAT;
            uint8_t l = lens[p * kK + k];
            if (l < 1 || l > kMaxLen) return ECCO_EFORMAT;
            kraft += 1u << (kMaxLen - l);
        }
        if (kraft != (1u << kMaxLen)) return ECCO_EFORMAT;  // complete prefix code required
    }
    return ECCO_OK;
}

// canonical order of pattern p's symbols: by (length, symbol)
static void canonical_order(const uint8_t* lens, int* order) {
    int n = 0;
    for (int l = 1; l <= kMaxLen; ++l)
        for (int k = 0; k < kK; ++k)
            if (lens[k] == l) order[n++] = k;
}

void derive_codes(ecco_model* m) {
    for (int p = 0; p < m->S; ++p) {
        const uint8_t* l = &m->lens[p * kK];
        int order[kK];
        canonical_order(l, order);
        uint32_t code = 0;
        for (int j = 0; j < kK; ++j) {
            if (j) code = (code + 1) << (l[order[j]] - l[order[j - 1]]);
            m->codes[p * kK + order[j]] = (uint16_t)code;
        }
    }
    m->max_len = 0;
    for (int i = 0; i < m->S * kK; ++i) m->max_len = std::max<int>(m->max_len, m->lens[i]);
}

void build_device_image(const ecco_model* m, uint32_t* img) {
    const DevLayout D{m->S};
    std::memset(img, 0, D.image_words() * 4);
    uint32_t* enc = img + D.enc();
    uint32_t* longtab = img + D.longtab();
    std::memcpy(img + D.cent(), m->cent, sizeof(uint16_t) * m->S * kK);
    for (int p = 0; p < m->S; ++p) {
        int order[kK];
        canonical_order(&m->lens[p * kK], order);
        for (int j = 0; j < kK; ++j) {
            int k = order[j], l = m->lens[p * kK + k];
            longtab[p * kK + j] = ((uint32_t)m->codes[p * kK + k] << (kMaxLen - l)) | ((uint32_t)k << 12) | ((uint32_t)l << 16);
        }
        for (int k = 0; k < kK; ++k) enc[p * kK + k] = (uint32_t)m->codes[p * kK + k] | ((uint32_t)m->lens[p * kK + k] << 16);
    }
}

}  // namespace ecco

using namespace ecco;

namespace {
constexpr uint32_t kMagic = 0x30434345u;  // "ECC0"
struct Header { uint32_t magic, version, S, K; };
}  // namespace

extern "C" {

const char* ecco_strerror(int status) {
    switch (status) {
        case ECCO_OK: return "ok";
        case ECCO_EINVAL: return "invalid argument";
        case ECCO_ESHAPE: return "invalid shape";
        case ECCO_EALIGN: return "misaligned pointer";
        case ECCO_ENOMEM: return "out of memory";
        case ECCO_EFORMAT: return "model fails validation";
        case ECCO_EHIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int ecco_model_create(const uint16_t* centroids, const uint8_t* code_lens, int S, ecco_model** out) {
    if (!centroids || !code_lens || !out) return ECCO_EINVAL;
    if (S < 1 || S > kMaxS) return ECCO_EINVAL;
    int rc = validate_tables(centroids, code_lens, S);
    if (rc != ECCO_OK) return rc;
    ecco_model* m = new (std::nothrow) ecco_model;
    if (!m) return ECCO_ENOMEM;
    m->S = S;
    std::memcpy(m->cent, centroids, sizeof(uint16_t) * S * kK);
    std::memcpy(m->lens, code_lens, (size_t)S * kK);
    derive_codes(m);
    *out = m;
    return ECCO_OK;
}

int ecco_model_save(const ecco_model* m, void* buf, size_t cap, size_t* written) {
    if (!m || !written) return ECCO_EINVAL;
    size_t need = sizeof(Header) + (size_t)m->S * kK * 3;
    *written = need;
    if (!buf) return ECCO_OK;
    if (cap < need) return ECCO_EINVAL;
    Header h{kMagic, 1u, (uint32_t)m->S, (uint32_t)kK};
    unsigned char* p = static_cast<unsigned char*>(buf);
    std::memcpy(p, &h, sizeof h);
    std::memcpy(p + sizeof h, m->cent, (size_t)m->S * kK * 2);
    std::memcpy(p + sizeof h + (size_t)m->S * kK * 2, m->lens, (size_t)m->S * kK);
    return ECCO_OK;
}

int ecco_model_load(const void* buf, size_t len, ecco_model** out) {
    if (!buf || !out) return ECCO_EINVAL;
    if (len < sizeof(Header)) return ECCO_EFORMAT;
    Header h;
    std::memcpy(&h, buf, sizeof h);
    if (h.magic != kMagic || h.version != 1u || h.K != (uint32_t)kK || h.S < 1 || h.S > (uint32_t)kMaxS) return ECCO_EFORMAT;
    size_t need = sizeof(Header) + (size_t)h.S * kK * 3;
    if (len != need) return ECCO_EFORMAT;
    const unsigned char* p = static_cast<const unsigned char*>(buf) + sizeof h;
    std::vector<uint16_t> cent((size_t)h.S * kK);
    std::memcpy(cent.data(), p, cent.size() * 2);
    return ecco_model_create(cent.data(), p + cent.size() * 2, (int)h.S, out);
}

int ecco_model_S(const ecco_model* m) { return m ? m->S : 0; }
const uint16_t* ecco_model_centroids(const ecco_model* m) { return m ? m->cent : nullptr; }
const uint8_t* ecco_model_code_lens(const ecco_model* m) { return m ? m->lens : nullptr; }

int ecco_model_to_device(ecco_model* m, int device) {
    if (!m || device < 0) return ECCO_EINVAL;
    if (m->dev && m->device == device) return ECCO_OK;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device >= count) return ECCO_EHIP;
    int prev = 0;
    if (hipGetDevice(&prev) != hipSuccess) return ECCO_EHIP;
    if (m->dev) {
        (void)hipSetDevice(m->device);
        (void)hipFree(m->dev);
        m->dev = nullptr;
        m->device = -1;
    }
    if (hipSetDevice(device) != hipSuccess) return ECCO_EHIP;
    const DevLayout D{m->S};
    std::vector<uint32_t> img(D.image_words());
    build_device_image(m, img.data());
    void* d = nullptr;
    hipError_t e = hipMalloc(&d, D.total_bytes());
    if (e != hipSuccess) {
        (void)hipSetDevice(prev);
        return e == hipErrorOutOfMemory ? ECCO_ENOMEM : ECCO_EHIP;
    }
    e = hipMemcpy(d, img.data(), D.image_words() * 4, hipMemcpyHostToDevice);
    const int scratch_rc = init_device_scratch(device);  // while `device` is current
    (void)hipSetDevice(prev);
    if (e != hipSuccess || scratch_rc != ECCO_OK) {
        (void)hipFree(d);
        return ECCO_EHIP;
    }
    m->dev = static_cast<uint32_t*>(d);
    m->device = device;
    return ECCO_OK;
}

void ecco_model_free(ecco_model* m) {
    if (!m) return;
    if (m->dev) {
        int prev = 0;
        if (hipGetDevice(&prev) == hipSuccess) {
            (void)hipSetDevice(m->device);
            (void)hipFree(m->dev);
            (void)hipSetDevice(prev);
        }
    }
    delete m;
}

}  // extern "C"
