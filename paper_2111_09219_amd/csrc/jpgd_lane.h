// What one lane does: decode JPEG syntax elements from an arbitrary bit position and decoder state
// (paper, Algorithm 2 "decode_subsequence" and the function decode_next_symbol it calls).
// Host/device code: the kernels inline it, and a host build of the same functions is exercised
// on the CPU by the test suite.
#pragma once
#include "jpgd_common.h"

namespace jpgd {

// Decoder state of the paper, (p, n, c, z), with c refined to the data unit inside the MCU
// (two decoders inside different luminance units of a 4:2:0 MCU agree on the component but
// not on what follows) and n kept as completed data units (see SInfo).
struct Lane {
    uint32_t p;    // bit position in the unstuffed stream of the next syntax element
    uint32_t u4;   // 4 * (data unit inside the MCU)
    uint32_t z;    // zig-zag index of the next coefficient (0 = a DC symbol is next)
    uint32_t nb;   // data units completed since the counter was last cleared
};

// 64-bit window on the stream, most significant bit first; at least 32 bits are valid before
// every symbol (a codeword has at most 16 bits, its value at most 16).
struct BitWin {
    uint64_t bb;
    int32_t cnt;     // valid bits in bb
    uint32_t next;   // cursor of the next 32-bit word, in the units of the Fetch functor
};

// per-image constants of the scan syntax
struct Syntax {
    uint32_t sched_dc, sched_ac, sched_comp;  // 4 bits per data unit (see ImgDesc)
    uint32_t upm4;                            // 4 * units per MCU
};

// `cursor` addresses the 32-bit word that holds bit p
template <class Fetch>
JPGD_HD void win_init(BitWin& w, uint32_t p, uint32_t cursor, Fetch fetch) {
    uint32_t o = p & 31u;
    uint64_t v = ((uint64_t)fetch(cursor) << 32) | (uint64_t)fetch(cursor + 1u);
    w.bb = v << o;
    w.cnt = 64 - (int32_t)o;
    w.next = cursor + 2u;
    if (w.cnt <= 32) {
        w.bb |= (uint64_t)fetch(w.next) << (32 - w.cnt);
        w.cnt += 32;
        w.next++;
    }
}

// table entry for the symbol at the head of `peek` (see jpgd_common.h for the format)
template <class LutPtr>
JPGD_HD uint32_t lookup(uint32_t peek, bool is_dc, uint32_t u4, const Syntax& sx, LutPtr lut) {
    uint32_t sched = is_dc ? sx.sched_dc : sx.sched_ac;
    uint32_t base = ((sched >> u4) & 15u) * (uint32_t)kLutEntries;
    uint32_t e = lut[base + (peek >> (32 - kLutK))];
    if (lut_len(e) == 0u) {  // codeword longer than kLutK bits, or none at all
        uint32_t nb2 = (e >> 5) & 7u, off = (e >> 8) << 1;
        uint32_t j = (peek >> (32 - kLutK - nb2)) & ((1u << nb2) - 1u);
        e = lut[base + (uint32_t)kLutL1 + off + j];
    }
    return e;
}

// value bits follow the codeword; "signed ones' complement" (paper, Section 2): a leading 1 means the
// bits are the value itself, a leading 0 means value = bits - (2^size - 1); size 0 gives 0
JPGD_HD int32_t symbol_value(uint32_t peek, uint32_t len, uint32_t size) {
    uint32_t t = peek << len;
    uint32_t v = size ? (t >> (32u - size)) : 0u;
    uint32_t ones = (1u << size) - 1u;
    return (int32_t)v - (int32_t)((int32_t)t < 0 ? 0u : ones);
}

// Advances (z, u, nb) by the slots a symbol covers (paper, Algorithm 2: n, z += run_length + 1; z is
// reset when the unit is complete and the next unit begins).  Returns true when the unit was completed.
JPGD_HD bool advance(Lane& l, uint32_t adv, const Syntax& sx) {
    uint32_t zn = l.z + adv;
    bool done = zn >= 64u;
    l.z = done ? 0u : zn;
    uint32_t un = l.u4 + 4u;
    un = un == sx.upm4 ? 0u : un;
    l.u4 = done ? un : l.u4;
    l.nb += done ? 1u : 0u;
    return done;
}

template <class Fetch>
JPGD_HD void consume(Lane& l, BitWin& w, uint32_t total, Fetch fetch) {
    total = total ? total : 1u;  // every table entry has a length of at least one bit; never stand still
    w.bb <<= total;
    w.cnt -= (int32_t)total;
    l.p += total;
    if (w.cnt <= 32) {
        w.bb |= (uint64_t)fetch(w.next) << (32 - w.cnt);
        w.cnt += 32;
        w.next++;
    }
}

// DC-difference sums of the three components, kept in one 64-bit accumulator with 15-bit fields
// (component c at bit 15*c) so that a single multiply-add updates the right one.  A subsequence's
// true sums are differences of two quantised DC values and fit easily; sums of lanes that are not
// synchronised may spill into the neighbouring field, and are discarded anyway.
JPGD_HD void dc_unpack(int64_t acc, int32_t& d0, int32_t& d1, int32_t& d2) {
    d0 = (int32_t)((int64_t)((uint64_t)acc << 49) >> 49);
    acc = (acc - d0) >> 15;
    d1 = (int32_t)((int64_t)((uint64_t)acc << 49) >> 49);
    acc = (acc - d1) >> 15;
    d2 = (int32_t)acc;
}

// Synchronisation pass (write = false in Algorithm 2): decode while the next symbol starts before
// `limit`, keeping the state, the count of completed units and the per-component DC sums.
template <class Fetch, class LutPtr>
JPGD_HD void decode_span_sync(Lane& l, BitWin& w, uint32_t limit, int64_t& dcacc, const Syntax& sx, Fetch fetch,
                              LutPtr lut) {
    while (l.p < limit) {
        const uint32_t peek = (uint32_t)(w.bb >> 32);
        const bool is_dc = l.z == 0u;
        const uint32_t e = lookup(peek, is_dc, l.u4, sx, lut);
        const uint32_t len = lut_len(e), size = lut_size(e);
        const int32_t d = is_dc ? symbol_value(peek, len, size) : 0;
        const uint32_t comp = (sx.sched_comp >> l.u4) & 15u;
        dcacc += (int64_t)d * (int64_t)(int32_t)(1u << (15u * comp));
        advance(l, lut_adv(e), sx);
        consume(l, w, len + size, fetch);
    }
}

// Write pass (write = true in Algorithm 2): the same walk, storing every non-zero coefficient at
// 64*unit + zig-zag index, DC values un-differenced.  `unit` is the index of the data unit being
// decoded, `total_units` the end of the image, pred[] the DC predictors; `flags` collects kSt* bits.
template <class Fetch, class LutPtr, class Store>
JPGD_HD void decode_span_write(Lane& l, BitWin& w, uint32_t limit, uint32_t& unit, uint32_t total_units,
                               int32_t& pred0, int32_t& pred1, int32_t& pred2, const Syntax& sx, Fetch fetch,
                               LutPtr lut, Store store, uint32_t& flags) {
    while (l.p < limit && unit < total_units) {
        const uint32_t peek = (uint32_t)(w.bb >> 32);
        const bool is_dc = l.z == 0u;
        const uint32_t e = lookup(peek, is_dc, l.u4, sx, lut);
        const uint32_t len = lut_len(e), size = lut_size(e), adv = lut_adv(e);
        const int32_t value = symbol_value(peek, len, size);
        if (adv == 0u) flags |= kStInvalid;  // no codeword
        if (is_dc) {
            const uint32_t comp = (sx.sched_comp >> l.u4) & 15u;
            int32_t pred = comp == 0u ? pred0 : (comp == 1u ? pred1 : pred2);
            pred += value;
            pred0 = comp == 0u ? pred : pred0;
            pred1 = comp == 1u ? pred : pred1;
            pred2 = comp == 2u ? pred : pred2;
            if (adv) store(unit, 0u, (int16_t)pred);
        } else if (size) {
            const uint32_t at = l.z + adv - 1u;  // after the run of zeros
            if (at < 64u) store(unit, at, (int16_t)value);
            else flags |= kStInvalid;
        } else if (adv == 16u && l.z + 16u > 64u) {
            flags |= kStInvalid;  // ZRL running past the end of the unit
        }
        if (advance(l, adv, sx)) unit++;
        consume(l, w, len + size, fetch);
    }
}

}  // namespace jpgd
