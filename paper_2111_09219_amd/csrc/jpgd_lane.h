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
    int32_t dc0, dc1, dc2;  // sync pass: sums of DC differences; write pass: DC predictors
};

// 64-bit window on the stream, most significant bit first; at least 32 bits are valid before
// every symbol (a codeword has at most 16 bits, its value at most 16).
struct BitWin {
    uint64_t bb;
    int32_t cnt;     // valid bits in bb
    uint32_t next;   // index of the next 32-bit word to fetch
};

// per-image constants of the scan syntax
struct Syntax {
    uint32_t sched_dc, sched_ac, sched_comp;  // 4 bits per data unit (see ImgDesc)
    uint32_t upm4;                            // 4 * units per MCU
};

template <class Fetch>
JPGD_HD void win_init(BitWin& w, uint32_t p, Fetch fetch) {
    uint32_t i = p >> 5, o = p & 31u;
    uint64_t v = ((uint64_t)fetch(i) << 32) | (uint64_t)fetch(i + 1);
    w.bb = v << o;
    w.cnt = 64 - (int32_t)o;
    w.next = i + 2;
    if (w.cnt <= 32) {
        w.bb |= (uint64_t)fetch(w.next) << (32 - w.cnt);
        w.cnt += 32;
        w.next++;
    }
}

// Result of looking one symbol up; lookup is separated from the state update so that the sync pass
// and the write pass share it.
struct Sym {
    uint32_t len;    // codeword bits
    uint32_t size;   // value bits
    uint32_t run;    // zeros before the coefficient
    bool eob;        // end of block (or a zero-size symbol treated as one)
    bool nop;        // no codeword matched: one bit is skipped and nothing else changes
    int32_t value;   // decoded coefficient or DC difference (0 when size == 0)
};

template <class LutPtr>
JPGD_HD Sym lookup(uint32_t peek, bool is_dc, uint32_t u4, const Syntax& sx, LutPtr lut) {
    uint32_t sched = is_dc ? sx.sched_dc : sx.sched_ac;
    uint32_t base = ((sched >> u4) & 15u) * (uint32_t)kLutEntries;
    uint32_t e = lut[base + (peek >> (32 - kLutK))];
    Sym s;
    s.nop = false;
    if (e & kLutEscape) {
        uint32_t nb2 = (e >> 9) & 7u, off = e & 511u;
        uint32_t j = (peek >> (32 - kLutK - nb2)) & ((1u << nb2) - 1u);
        e = lut[base + kLutL1 + off + j];
        s.nop = (e & kLutNop) != 0;
    }
    s.len = e & 31u;
    s.size = (e >> 5) & 31u;
    s.run = (e >> 10) & 15u;
    s.eob = (e & kLutEob) != 0;
    // value bits follow the codeword; "signed ones' complement" (paper, Section 2): a leading 1 means
    // the bits are the value itself, a leading 0 means value = bits - (2^size - 1)
    uint32_t t = peek << s.len;
    uint32_t v = s.size ? (t >> (32 - s.size)) : 0u;
    int32_t lead = (int32_t)t >> 31;  // all ones if the first value bit is 1
    s.value = (int32_t)v - (int32_t)(~(uint32_t)lead & ((1u << s.size) - 1u));
    return s;
}

// Advances (z, u, nb) past a symbol: run+1 slots for a coefficient, 16 for ZRL, the rest of the unit
// for EOB (paper, Algorithm 2: n, z += run_length + 1; z reset when the unit is complete; next unit).
// Returns true when the unit was completed.
JPGD_HD bool advance(Lane& l, const Sym& s, const Syntax& sx) {
    uint32_t adv = s.eob ? 64u - l.z : s.run + 1u;
    adv = s.nop ? 0u : adv;
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

// Synchronisation pass (write = false in Algorithm 2): decode while the next symbol starts before
// `limit`, keeping the state, the count of completed units and the per-component DC sums.
template <class Fetch, class LutPtr>
JPGD_HD void decode_span_sync(Lane& l, BitWin& w, uint32_t limit, const Syntax& sx, Fetch fetch, LutPtr lut) {
    while (l.p < limit) {
        uint32_t peek = (uint32_t)(w.bb >> 32);
        bool is_dc = l.z == 0u;
        Sym s = lookup(peek, is_dc, l.u4, sx, lut);
        uint32_t comp = (sx.sched_comp >> l.u4) & 15u;
        int32_t d = is_dc ? s.value : 0;
        l.dc0 += comp == 0u ? d : 0;
        l.dc1 += comp == 1u ? d : 0;
        l.dc2 += comp == 2u ? d : 0;
        advance(l, s, sx);
        consume(l, w, s.len + s.size, fetch);
    }
}

// Write pass (write = true in Algorithm 2): the same walk, storing every non-zero coefficient at
// 64*unit + zig-zag index, DC values un-differenced.  `unit` is the index of the data unit being
// decoded, `total_units` the end of the image; `flags` collects kSt* bits.
template <class Fetch, class LutPtr, class Store>
JPGD_HD void decode_span_write(Lane& l, BitWin& w, uint32_t limit, uint32_t& unit, uint32_t total_units,
                               const Syntax& sx, Fetch fetch, LutPtr lut, Store store, uint32_t& flags) {
    while (l.p < limit && unit < total_units) {
        uint32_t peek = (uint32_t)(w.bb >> 32);
        bool is_dc = l.z == 0u;
        Sym s = lookup(peek, is_dc, l.u4, sx, lut);
        if (s.nop) flags |= kStInvalid;
        if (is_dc) {
            uint32_t comp = (sx.sched_comp >> l.u4) & 15u;
            int32_t pred = comp == 0u ? l.dc0 : (comp == 1u ? l.dc1 : l.dc2);
            pred += s.value;
            l.dc0 = comp == 0u ? pred : l.dc0;
            l.dc1 = comp == 1u ? pred : l.dc1;
            l.dc2 = comp == 2u ? pred : l.dc2;
            if (!s.nop) store(unit, 0u, (int16_t)pred);
        } else if (s.size) {
            uint32_t at = l.z + s.run;
            if (at < 64u) store(unit, at, (int16_t)s.value);
            else flags |= kStInvalid;
        } else if (!s.eob && !s.nop && l.z + 16u > 64u) {
            flags |= kStInvalid;  // ZRL running past the end of the unit
        }
        if (advance(l, s, sx)) unit++;
        consume(l, w, s.len + s.size, fetch);
    }
}

}  // namespace jpgd
