// Host-side construction of the two-level Huffman lookup tables the kernels keep in LDS.
// Layout and entry format: jpgd_common.h.
#pragma once
#include <string.h>

#include "jpgd_common.h"

namespace jpgd {

// bits[l-1] = number of codes of length l, vals = symbols in code order (as stored in a DHT segment).
// Codewords are assigned canonically: shortest first, in list order, counting upward, the running
// code doubled whenever the length grows.  Returns false if the lists cannot be a prefix code.
inline bool build_lut(const uint8_t bits[16], const uint8_t* vals, bool is_dc, uint16_t* out) {
    uint32_t first[17], count[17], valptr[17];
    uint32_t code = 0, k = 0;
    for (int len = 1; len <= 16; ++len) {
        first[len] = code;
        count[len] = bits[len - 1];
        valptr[len] = k;
        code += count[len];
        k += count[len];
        if (code > (1u << len)) return false;
        code <<= 1;
    }
    if (k > 256) return false;
    if (is_dc)
        for (uint32_t i = 0; i < k; ++i)
            if (vals[i] > 11) return false;  // a DC symbol is a number of value bits: 0..11 for 8-bit samples

    auto entry_for = [&](uint32_t sym, int len) -> uint16_t {
        uint32_t size, adv;
        if (is_dc) {
            size = sym;  // at most 11, checked above
            adv = 1;
        } else {
            uint32_t run = sym >> 4;
            size = sym & 15;
            adv = size ? run + 1 : (run == 15 ? 16u : kAdvEob);
        }
        return (uint16_t)(((uint32_t)len + size) | (size << 5) | (adv << 9));
    };

    const uint16_t kUnset = 0xFFFF;
    for (int i = 0; i < kLutL1; ++i) out[i] = kUnset;
    uint8_t maxlen[kLutL1];
    memset(maxlen, 0, sizeof maxlen);
    for (int len = 1; len <= 16; ++len)
        for (uint32_t i = 0; i < count[len]; ++i) {
            uint32_t c = first[len] + i;
            if (len <= kLutK) {
                uint16_t e = entry_for(vals[valptr[len] + i], len);
                uint32_t lo = c << (kLutK - len), n = 1u << (kLutK - len);
                for (uint32_t j = 0; j < n; ++j) out[lo + j] = e;
            } else {
                uint32_t prefix = c >> (len - kLutK);
                if (maxlen[prefix] < len) maxlen[prefix] = (uint8_t)len;
            }
        }
    // second level: entries 0 and 1 are the shared "no codeword" record (one bit, nothing else), then one
    // subtable per escaping prefix; subtables hold 2, 4, .. 64 entries, so every offset is even
    uint16_t* l2 = out + kLutL1;
    const uint16_t invalid = 1u;
    for (int i = 0; i < kLutL2; ++i) l2[i] = invalid;
    uint32_t used = 2;
    uint32_t suboff[kLutL1];
    for (int p = 0; p < kLutL1; ++p) {
        if (maxlen[p]) {
            if (out[p] != kUnset) return false;  // a short code is a prefix of a long one
            uint32_t nb2 = maxlen[p] - kLutK, n = 1u << nb2;
            if (used + n > (uint32_t)kLutL2) return false;
            suboff[p] = used;
            out[p] = (uint16_t)(0x8000u | nb2 | ((used >> 1) << 3));
            used += n;
        } else if (out[p] == kUnset) {
            out[p] = 0x8000u;  // escape with zero further bits and offset 0: the invalid record
        }
    }
    for (int len = kLutK + 1; len <= 16; ++len)
        for (uint32_t i = 0; i < count[len]; ++i) {
            uint32_t c = first[len] + i;
            uint32_t prefix = c >> (len - kLutK);
            uint32_t ml = maxlen[prefix];
            uint32_t low = c & ((1u << (len - kLutK)) - 1u);
            uint32_t lo = low << (ml - len), n = 1u << (ml - len);
            uint16_t e = entry_for(vals[valptr[len] + i], len);
            for (uint32_t j = 0; j < n; ++j) l2[suboff[prefix] + lo + j] = e;
        }
    return true;
}

// Pair bytes of an AC table (synchronisation pass, two symbols per step): for first-level index i, if the entry is
// a coefficient or a run of sixteen zeros that takes t1 < kLutK bits and the rest of the index holds the whole
// codeword of another symbol of the table -- taking t2 <= 15 bits with its value bits, covering at most 14 slots
// or being end-of-block -- the byte is t2 | c << 4 with c = slots covered, 15 for end-of-block; otherwise 0.
// lut: the table's kLutEntries entries (build_lut); pairs: kPairBytes bytes.
inline void build_pairs(const uint16_t* lut, uint8_t* pairs) {
    for (uint32_t i = 0; i < (uint32_t)kLutL1; ++i) {
        pairs[i] = 0;
        const uint32_t e1 = lut[i];
        if (lut_esc(e1)) continue;
        const uint32_t a1 = lut_adv(e1), t1 = lut_total(e1);
        if (a1 == 0u || a1 == kAdvEob || t1 >= (uint32_t)kLutK) continue;
        const uint32_t e2 = lut[(i << t1) & (uint32_t)(kLutL1 - 1)];  // the bits behind the first symbol, zeros appended
        if (lut_esc(e2)) continue;
        const uint32_t t2 = lut_total(e2), a2 = lut_adv(e2);
        if (t2 - lut_size(e2) > (uint32_t)kLutK - t1) continue;        // the codeword reaches beyond the index
        if (a2 == 0u || t2 > 15u || (a2 != kAdvEob && a2 > 14u)) continue;
        pairs[i] = (uint8_t)(t2 | ((a2 == kAdvEob ? 15u : a2) << 4));
    }
}

}  // namespace jpgd
