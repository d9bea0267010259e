// Runs the CPU-side code of the repository -- the oracle, the input encoder, the product's header parser and table
// builder, and the host walk-through of the kernels' lane code -- under AddressSanitizer and
// UndefinedBehaviorSanitizer: intact files of every layout (also extreme shapes), damaged entropy-coded data,
// truncated and mutated headers.  Built and run by tests/test_sanitizers.py; test code only.
//
// Exit status 0 = every case ran clean and, where both decoders accept a file, their coefficients agree.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/jpgd.h"

extern "C" {
// workloads/jpeg_encoder.c
int wl_encode_jpeg(const uint8_t* pixels, int width, int height, int ncomp, int subsampling, int quality, int optimize,
                   int restart_interval, uint8_t** out_file, size_t* out_len, int16_t* out_coef, size_t* scan_offset,
                   size_t* scan_len);
void wl_free(void* p);
// oracle/jpeg_oracle.c (opaque handle; sizes are asked through jpgd_parse, which the tests pin to the oracle's parser)
int orc_open(const uint8_t* file, size_t len, void** out);
void orc_close(void* im);
int orc_decode_coefficients(const void* im, int16_t* coef, int64_t* end_bit);
int orc_decode_pixels(const void* im, const int16_t* coef, uint8_t* pixels);
int orc_decode_planes(const void* im, const int16_t* coef, uint8_t* planes);
int orc_decode_pixels_scaled(const void* im, const int16_t* coef, int d, uint8_t* pixels);
int orc_decode_planes_scaled(const void* im, const int16_t* coef, int d, uint8_t* planes);
int64_t orc_unstuffed_len(const void* im);
int orc_boundary_states(const void* im, int L, int64_t nsub, int64_t* p, int32_t* u, int32_t* z, int32_t* units,
                        int64_t* slots, int32_t* dcsum, int32_t* restart);
// tests/emul/jpgd_emul.cpp
int emul_decode(const uint8_t* file, size_t len, uint32_t L, uint32_t H, uint32_t max_rounds, int16_t* coef, uint8_t* pix,
                uint32_t* sinfo_out, uint32_t sinfo_cap, uint8_t* stream_out, uint32_t* stats);
void emul_set_coop_max(uint32_t n);
}

static uint64_t g_rng = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() {
    g_rng ^= g_rng << 13; g_rng ^= g_rng >> 7; g_rng ^= g_rng << 17;
    return (uint32_t)(g_rng >> 32);
}

static std::vector<uint8_t> make_pixels(int w, int h, int ncomp, int noise) {
    std::vector<uint8_t> px((size_t)w * h * ncomp);
    for (int y = 0; y < h; ++y)
        for (int x = 0; x < w; ++x)
            for (int c = 0; c < ncomp; ++c) {
                int v = (x * 3 + y * 2 + c * 40) % 256 + (noise ? (int)(rnd() % (2u * noise + 1u)) - noise : 0);
                if (((x / 16) + (y / 16)) % 5 == 0) v = 255 - v;  // some edges
                px[((size_t)y * w + x) * ncomp + c] = (uint8_t)(v < 0 ? 0 : v > 255 ? 255 : v);
            }
    return px;
}

static int failures = 0;
#define CHECK(cond, ...)                                  \
    do {                                                  \
        if (!(cond)) {                                    \
            fprintf(stderr, "san_driver: " __VA_ARGS__);  \
            fprintf(stderr, "\n");                        \
            ++failures;                                   \
        }                                                 \
    } while (0)

// decodes one file with the oracle and with the walk-through; returns 1 if both accepted it
static int decode_both(const std::vector<uint8_t>& file, uint32_t L, uint32_t H, bool all_outputs) {
    jpgd_info info;
    const int prc = jpgd_parse(file.data(), file.size(), &info);
    void* im = nullptr;
    const int orc = orc_open(file.data(), file.size(), &im);
    if (prc != JPGD_OK || orc != 0) {
        if (im) orc_close(im);
        return 0;
    }
    const size_t units = info.total_units;
    std::vector<int16_t> ref(units * 64), got(units * 64);
    std::vector<uint8_t> pix((size_t)info.width * info.height * info.ncomp + 16), pix2(pix.size());
    const int rc_o = orc_decode_coefficients(im, ref.data(), nullptr);
    uint32_t stats[8] = {0};
    const int rc_e = emul_decode(file.data(), file.size(), L, H, 64, got.data(), pix2.data(), nullptr, 0, nullptr, stats);
    CHECK(rc_e == JPGD_OK || rc_e == JPGD_E_CORRUPT, "walk-through returned %d", rc_e);
    int both = 0;
    if (rc_o == 0 && rc_e == JPGD_OK) {
        both = 1;
        CHECK(memcmp(ref.data(), got.data(), ref.size() * 2) == 0, "coefficients differ (%ux%u, L=%u H=%u)", info.width,
              info.height, L, H);
    }
    if (rc_o == 0 && all_outputs) {
        CHECK(orc_decode_pixels(im, ref.data(), pix.data()) == 0, "orc_decode_pixels");
        CHECK(orc_decode_planes(im, ref.data(), pix.data()) == 0, "orc_decode_planes");
        for (int d = 2; d <= 8; d *= 2) {
            CHECK(orc_decode_pixels_scaled(im, ref.data(), d, pix.data()) == 0, "orc_decode_pixels_scaled");
            CHECK(orc_decode_planes_scaled(im, ref.data(), d, pix.data()) == 0, "orc_decode_planes_scaled");
        }
        const int64_t nbytes = orc_unstuffed_len(im);
        const int64_t nsub = (nbytes * 8 + L - 1) / L > 0 ? (nbytes * 8 + L - 1) / L : 1;
        std::vector<int64_t> p(nsub), slots(nsub);
        std::vector<int32_t> u(nsub), z(nsub), un(nsub), dc(3 * nsub), rs(nsub);
        CHECK(orc_boundary_states(im, (int)L, nsub, p.data(), u.data(), z.data(), un.data(), slots.data(), dc.data(), rs.data()) == 0,
              "orc_boundary_states");
    }
    orc_close(im);
    return both;
}

static std::vector<uint8_t> encode(const std::vector<uint8_t>& px, int w, int h, int ncomp, int sub, int q, int opt, int ri,
                                   size_t* so, size_t* sl) {
    uint8_t* out = nullptr;
    size_t n = 0;
    std::vector<int16_t> coef;
    const int rc = wl_encode_jpeg(px.data(), w, h, ncomp, sub, q, opt, ri, &out, &n, nullptr, so, sl);
    if (rc != 0 || !out) {
        fprintf(stderr, "san_driver: encoder refused %dx%d\n", w, h);
        exit(2);
    }
    std::vector<uint8_t> file(out, out + n);
    wl_free(out);
    return file;
}

int main() {
    struct Case { int w, h, ncomp, sub, q, opt, ri; };
    const Case cases[] = {
        {51, 37, 1, 0, 85, 0, 0},   {333, 200, 3, 0, 94, 1, 0},   {8, 8, 3, 2, 40, 0, 0},     {70, 129, 3, 1, 75, 1, 3},
        {1, 1, 3, 0, 90, 0, 0},     {65535, 9, 1, 0, 80, 0, 0},   {9, 6001, 3, 2, 80, 0, 0},  {5000, 3, 3, 1, 80, 0, 1},
        {231, 153, 3, 2, 100, 0, 0}, {120, 72, 3, 2, 85, 0, 1},   {96, 64, 3, 0, 85, 0, 4},   {200, 150, 3, 2, 97, 1, 17},
    };
    int accepted = 0, cases_run = 0;
    for (const Case& c : cases) {
        const std::vector<uint8_t> px = make_pixels(c.w, c.h, c.ncomp, c.q >= 97 ? 60 : 8);
        size_t so = 0, sl = 0;
        const std::vector<uint8_t> file = encode(px, c.w, c.h, c.ncomp, c.sub, c.q, c.opt, c.ri, &so, &sl);
        const uint32_t Ls[3] = {128u, 256u, 1024u}, Hs[3] = {16u, 0u, 32u}, coop[3] = {6u, 64u, 0u};
        for (int k = 0; k < 3; ++k) {
            emul_set_coop_max(coop[k]);
            const int ok = decode_both(file, Ls[k], Hs[k], k == 0);
            CHECK(ok == 1, "intact file %dx%d not decoded by both", c.w, c.h);
            ++cases_run;
        }
        // damaged entropy-coded data
        const bool small = (size_t)c.w * c.h <= 12000u;
        for (int trial = 0; trial < (small ? 24 : 3); ++trial) {
            std::vector<uint8_t> bad = file;
            const int hits = 1 + (int)(rnd() % 3u);
            for (int k = 0; k < hits && sl > 2; ++k) {
                const size_t pos = so + rnd() % sl;
                if (bad[pos] == 0xFF || bad[pos - 1] == 0xFF) continue;
                bad[pos] = (uint8_t)(rnd() % 255u);
            }
            emul_set_coop_max(coop[trial % 3]);
            accepted += decode_both(bad, Ls[trial % 3], Hs[trial % 3], trial % 5 == 0);
            ++cases_run;
        }
        if (small) {
            // truncated files and mutated headers: the two parsers must refuse or accept without touching anything
            // outside the buffer (each prefix is an allocation of exactly its length)
            for (size_t n = 0; n < file.size(); n += (n < so + 8 ? 3 : 211)) {
                std::vector<uint8_t> cut(file.begin(), file.begin() + n);
                decode_both(cut, 256u, 0u, false);
                ++cases_run;
            }
            for (int trial = 0; trial < 120; ++trial) {
                std::vector<uint8_t> bad = file;
                const size_t pos = rnd() % so;
                bad[pos] = (uint8_t)rnd();
                emul_set_coop_max(6u);
                decode_both(bad, 128u, 16u, trial % 7 == 0);
                ++cases_run;
            }
        }
    }
    printf("san_driver: %d cases, %d damaged streams accepted by both decoders, %d failures\n", cases_run, accepted, failures);
    return failures ? 1 : 0;
}
