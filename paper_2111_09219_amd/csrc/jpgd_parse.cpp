// jpgd_parse: marker-segment reader for baseline JPEG files.  Host only.
// (paper, Section 4.1: the batch is parsed and the Huffman tables extracted before any kernel runs)
#include <string.h>

#include "../../include/jpgd.h"

namespace {

inline unsigned be16(const uint8_t* p) { return ((unsigned)p[0] << 8) | p[1]; }

// a DHT list is usable if no length holds more codes than it has room for
bool table_is_prefix_code(const uint8_t bits[16]) {
    unsigned code = 0, total = 0;
    for (int len = 1; len <= 16; ++len) {
        code += bits[len - 1];
        total += bits[len - 1];
        if (code > (1u << len)) return false;
        code <<= 1;
    }
    return total >= 1 && total <= 256;
}

}  // namespace

extern "C" int jpgd_parse(const uint8_t* file, size_t len, jpgd_info* out) {
    if (!file || !out) return JPGD_E_ARG;
    memset(out, 0, sizeof *out);
    if (len < 4) return JPGD_E_TRUNCATED;
    if (file[0] != 0xFF || file[1] != 0xD8) return JPGD_E_MARKER;

    bool have_frame = false, have_scan = false;
    size_t pos = 2;
    while (!have_scan) {
        if (pos + 2 > len) return JPGD_E_TRUNCATED;
        if (file[pos] != 0xFF) return JPGD_E_MARKER;
        unsigned m = file[pos + 1];
        if (m == 0xFF) { pos += 1; continue; }                                 // fill byte
        if (m == 0x00) return JPGD_E_MARKER;
        if (m == 0x01 || (m >= 0xD0 && m <= 0xD8)) { pos += 2; continue; }     // stand-alone markers
        if (m == 0xD9) return JPGD_E_MARKER;                                   // image ends before a scan
        if (pos + 4 > len) return JPGD_E_TRUNCATED;
        unsigned seglen = be16(file + pos + 2);
        if (seglen < 2) return JPGD_E_MARKER;
        if (pos + 2 + seglen > len) return JPGD_E_TRUNCATED;
        const uint8_t* seg = file + pos + 4;
        unsigned n = seglen - 2;

        if (m == 0xC0) {
            if (have_frame) return JPGD_E_UNSUPPORTED;
            if (n < 6) return JPGD_E_TRUNCATED;
            if (seg[0] != 8) return JPGD_E_UNSUPPORTED;
            out->height = be16(seg + 1);
            out->width = be16(seg + 3);
            out->ncomp = seg[5];
            if (out->ncomp != 1 && out->ncomp != 3) return JPGD_E_UNSUPPORTED;
            if (out->height == 0 || out->width == 0) return JPGD_E_UNSUPPORTED;  // DNL-defined height
            if (n < 6 + 3 * out->ncomp) return JPGD_E_TRUNCATED;
            for (unsigned c = 0; c < out->ncomp; ++c) {
                out->hsamp[c] = seg[7 + 3 * c] >> 4;
                out->vsamp[c] = seg[7 + 3 * c] & 15;
                out->tq[c] = seg[8 + 3 * c];
                if (out->tq[c] > 3) return JPGD_E_TABLE;
            }
            have_frame = true;
        } else if (m >= 0xC1 && m <= 0xCF && m != 0xC4 && m != 0xC8) {
            return JPGD_E_UNSUPPORTED;  // extended, progressive, lossless, arithmetic (also DAC)
        } else if (m == 0xC4) {
            unsigned q = 0;
            while (q < n) {
                if (q + 17 > n) return JPGD_E_TRUNCATED;
                unsigned cls = seg[q] >> 4, id = seg[q] & 15;
                if (cls > 1 || id > 3) return JPGD_E_TABLE;
                const uint8_t* bits = seg + q + 1;
                if (!table_is_prefix_code(bits)) return JPGD_E_TABLE;
                unsigned total = 0;
                for (int i = 0; i < 16; ++i) total += bits[i];
                if (q + 17 + total > n) return JPGD_E_TRUNCATED;
                // A DC symbol is a count of value bits, 0..11 for the 8-bit samples of a baseline frame (T.81, F.1.2.1).
                // Larger counts cannot occur in a valid stream, and the kernels rely on the bound: a difference of
                // up to 11 bits keeps the per-subsequence DC sums inside their 15-bit fields.
                if (cls == 0)
                    for (unsigned i = 0; i < total; ++i)
                        if (seg[q + 17 + i] > 11) return JPGD_E_TABLE;
                memcpy(out->dht_bits[cls][id], bits, 16);
                memset(out->dht_vals[cls][id], 0, 256);
                memcpy(out->dht_vals[cls][id], seg + q + 17, total);
                out->dht_present[cls][id] = 1;
                q += 17 + total;
            }
        } else if (m == 0xDB) {
            unsigned q = 0;
            while (q < n) {
                unsigned prec = seg[q] >> 4, id = seg[q] & 15;
                if (prec > 1 || id > 3) return JPGD_E_TABLE;
                unsigned need = 1 + (prec ? 128 : 64);
                if (q + need > n) return JPGD_E_TRUNCATED;
                for (int i = 0; i < 64; ++i) {
                    unsigned v = prec ? be16(seg + q + 1 + 2 * i) : seg[q + 1 + i];
                    if (v == 0) return JPGD_E_TABLE;
                    out->qt[id][i] = (uint16_t)v;
                }
                out->qt_present[id] = 1;
                q += need;
            }
        } else if (m == 0xDD) {
            if (n < 2) return JPGD_E_TRUNCATED;
            out->restart_interval = be16(seg);
        } else if (m == 0xDA) {
            if (!have_frame) return JPGD_E_MARKER;
            if (n < 1) return JPGD_E_TRUNCATED;
            if (seg[0] != out->ncomp) return JPGD_E_UNSUPPORTED;  // one interleaved scan only
            if (n < 1 + 2 * out->ncomp + 3) return JPGD_E_TRUNCATED;
            for (unsigned c = 0; c < out->ncomp; ++c) {
                out->td[c] = seg[2 + 2 * c] >> 4;
                out->ta[c] = seg[2 + 2 * c] & 15;
                if (out->td[c] > 3 || out->ta[c] > 3) return JPGD_E_TABLE;
            }
            const uint8_t* tail = seg + 1 + 2 * out->ncomp;
            if (tail[0] != 0 || tail[1] != 63 || tail[2] != 0) return JPGD_E_UNSUPPORTED;  // spectral selection
            out->scan_offset = pos + 2 + seglen;
            have_scan = true;
        }
        pos += 2 + seglen;
    }

    if (out->ncomp == 1) {
        out->hsamp[0] = out->vsamp[0] = 1;  // a single component is never interleaved
    } else {
        bool ok = out->hsamp[1] == 1 && out->vsamp[1] == 1 && out->hsamp[2] == 1 && out->vsamp[2] == 1 &&
                  (out->hsamp[0] == 1 || out->hsamp[0] == 2) && (out->vsamp[0] == 1 || out->vsamp[0] == 2);
        if (!ok) return JPGD_E_UNSUPPORTED;
    }
    for (unsigned c = 0; c < out->ncomp; ++c) {
        if (!out->qt_present[out->tq[c]]) return JPGD_E_TABLE;
        if (!out->dht_present[0][out->td[c]] || !out->dht_present[1][out->ta[c]]) return JPGD_E_TABLE;
    }
    out->mcu_w = 8u * out->hsamp[0];
    out->mcu_h = 8u * out->vsamp[0];
    out->mcus_x = (out->width + out->mcu_w - 1) / out->mcu_w;
    out->mcus_y = (out->height + out->mcu_h - 1) / out->mcu_h;
    out->units_per_mcu = out->ncomp == 1 ? 1u : (unsigned)out->hsamp[0] * out->vsamp[0] + 2u;
    uint64_t units = (uint64_t)out->mcus_x * out->mcus_y * out->units_per_mcu;
    if (units > 0x3FFFFFFu) return JPGD_E_UNSUPPORTED;  // keeps 64*units inside 32 bits
    out->total_units = (uint32_t)units;

    // The entropy-coded bytes are not scanned here: they end where the last EOI marker of the file
    // starts (a 0xFF inside them is always followed by 0x00, never by 0xD9).
    size_t e = len;
    while (e >= out->scan_offset + 2 && !(file[e - 2] == 0xFF && file[e - 1] == 0xD9)) --e;
    if (e < out->scan_offset + 2) return JPGD_E_TRUNCATED;
    out->scan_bytes = (e - 2) - out->scan_offset;
    if (out->scan_bytes >= (1ull << 28)) return JPGD_E_UNSUPPORTED;  // bit positions are 32-bit
    return JPGD_OK;
}

extern "C" const char* jpgd_strerror(int status) {
    switch (status) {
        case JPGD_OK: return "ok";
        case JPGD_E_ARG: return "bad argument";
        case JPGD_E_TRUNCATED: return "file or segment truncated";
        case JPGD_E_MARKER: return "marker syntax error";
        case JPGD_E_UNSUPPORTED: return "outside the supported baseline subset";
        case JPGD_E_TABLE: return "missing or malformed table";
        case JPGD_E_CORRUPT: return "entropy-coded data inconsistent with the headers";
        case JPGD_E_WORKSPACE: return "workspace too small or misaligned";
        case JPGD_E_HIP: return "HIP runtime error";
        case JPGD_E_BUSY: return "too many calls in flight";
        default: return "unknown status";
    }
}

extern "C" int jpgd_abi_version(void) { return 2; }
