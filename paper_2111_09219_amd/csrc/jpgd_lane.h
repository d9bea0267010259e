// What one lane does: decode JPEG syntax elements from an arbitrary bit position and decoder state
// (paper, Algorithm 2 "decode_subsequence" and the function decode_next_symbol it calls).
// Host/device code: the kernels inline it, and a host build of the same functions is exercised
// on the CPU by the test suite.
//
// The loop is software-pipelined by hand.  One symbol depends on the previous one through a short
// chain -- table entry -> code + value length -> shifted window -> next table index -> LDS read -- and a
// lone wavefront spends most of its time waiting on that chain.  So the table entry of the NEXT
// symbol is requested as soon as the current entry has been unpacked, and everything that is not on
// the chain (DC sums, unit bookkeeping, stores, fetching stream words) is done while that read is in
// flight.  A codeword longer than the first-level index is resolved as an iteration of its own that
// consumes no bits, so the common path has no second dependent read.
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
    // derived from u4 (set_unit)
    uint32_t tb_ac;       // first entry of the unit's AC table inside the LUT array
    uint32_t tb_dc_next;  // first entry of the DC table of the unit that follows
    uint32_t comp;        // component of the unit
    // pipeline registers (prime)
    uint32_t e;           // table entry already read for the symbol at p (possibly a first-level escape)
    uint32_t base;        // table that entry came from
};

// 64-bit window on the stream, most significant bit first; at least 32 bits are valid before
// every symbol (a codeword has at most 16 bits, its value at most 16).
struct BitWin {
    uint64_t bb;
    int32_t cnt;     // valid bits in bb
    uint32_t next;   // cursor of the word held in `ahead`, in the units of the Fetch functor
    uint32_t ahead;  // the next 32-bit word, fetched one refill early so that its latency is hidden
};

// per-image constants of the scan syntax
struct Syntax {
    uint32_t sched_dc, sched_ac, sched_comp;  // 4 bits per data unit (see ImgDesc)
    uint32_t upm4;                            // 4 * units per MCU
};

JPGD_HD uint32_t next_unit(uint32_t u4, const Syntax& sx) {
    uint32_t un = u4 + 4u;
    return un == sx.upm4 ? 0u : un;
}

JPGD_HD void set_unit(Lane& l, const Syntax& sx) {
    l.tb_ac = ((sx.sched_ac >> l.u4) & 15u) * (uint32_t)kLutEntries;
    l.tb_dc_next = ((sx.sched_dc >> next_unit(l.u4, sx)) & 15u) * (uint32_t)kLutEntries;
    l.comp = (sx.sched_comp >> l.u4) & 15u;
}

// `cursor` addresses the 32-bit word that holds bit p
template <class Fetch>
JPGD_HD void win_init(BitWin& w, uint32_t p, uint32_t cursor, Fetch fetch) {
    uint32_t o = p & 31u;
    uint64_t v = ((uint64_t)fetch(cursor) << 32) | (uint64_t)fetch(cursor + 1u);
    w.bb = v << o;
    w.cnt = 64 - (int32_t)o;
    w.next = cursor + 2u;
    w.ahead = fetch(w.next);
    if (w.cnt <= 32) {
        w.bb |= (uint64_t)w.ahead << (32 - w.cnt);
        w.cnt += 32;
        w.next++;
        w.ahead = fetch(w.next);
    }
}

// Starts the pipeline: after (p, u4, z) and the window are set, read the entry of the symbol at p.
template <class LutPtr>
JPGD_HD void prime(Lane& l, const BitWin& w, const Syntax& sx, LutPtr lut) {
    set_unit(l, sx);
    const uint32_t tb_dc = ((sx.sched_dc >> l.u4) & 15u) * (uint32_t)kLutEntries;
    l.base = l.z == 0u ? tb_dc : l.tb_ac;
    l.e = lut[l.base + ((uint32_t)(w.bb >> 32) >> (32 - kLutK))];
}

// value bits follow the codeword; "signed ones' complement" (paper, Section 2): a leading 1 means the
// bits are the value itself, a leading 0 means value = bits - (2^size - 1), i.e. minus the complemented
// bits; size 0 gives 0
JPGD_HD int32_t symbol_value(uint32_t peek, uint32_t len, uint32_t size) {
    uint32_t t = peek << len;
    uint32_t m = (uint32_t)((int32_t)(~t) >> 31);   // all ones for a negative value
    // (t ^ m) >> (32 - size) without a special case for size 0: two shifts, the first by at least one
    uint32_t r = ((t ^ m) >> 1) >> (31u - size);
    return (int32_t)((r ^ m) - m);
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

// One step of the pipeline, shared by both passes.  Unpacks the entry in hand, moves the window and
// (z, u) past the symbol, and requests the entry of the next symbol (or, for an escape, the second-level
// entry of the same symbol).  What the passes do with the symbol itself comes after, in the shadow of
// that request.
struct Step {
    uint32_t peek;   // window as the symbol saw it
    uint32_t len, size, adv;
    bool esc;        // first-level escape: nothing was consumed, the state did not change
    bool is_dc;
    bool done;       // the symbol completed its data unit
    bool need;       // the window took the word in `ahead`; step_finish fetches the next one
    uint32_t z;      // zig-zag index the symbol started at
};

template <class LutPtr>
JPGD_HD Step step_and_request(Lane& l, BitWin& w, LutPtr lut) {
    Step s;
    const uint32_t e = l.e;
    s.peek = (uint32_t)(w.bb >> 32);
    s.len = lut_len(e);
    s.esc = s.len == 0u;
    s.size = s.esc ? 0u : lut_size(e);
    s.adv = s.esc ? 0u : lut_adv(e);
    s.is_dc = l.z == 0u;
    s.z = l.z;
    const uint32_t total = s.len + s.size;
    // window past the symbol; a word is taken from `ahead` when fewer than 33 bits remain
    w.bb <<= total;
    w.cnt -= (int32_t)total;
    s.need = w.cnt <= 32;
    const uint64_t more = (uint64_t)w.ahead << ((32 - w.cnt) & 63);
    w.bb |= s.need ? more : 0ull;
    w.cnt += s.need ? 32 : 0;
    // (z, u) past the symbol
    const uint32_t zn = l.z + s.adv;
    s.done = zn >= 64u;
    l.z = s.done ? 0u : zn;
    // request: next symbol from the DC table of the next unit or the AC table of this one; an escape asks
    // the second level of the table it came from
    const uint32_t peek2 = (uint32_t)(w.bb >> 32);
    const uint32_t base2 = s.done ? l.tb_dc_next : l.tb_ac;
    const uint32_t nb2 = (e >> 5) & 7u;
    const uint32_t sub = (uint32_t)kLutL1 + ((e >> 8) << 1) + ((s.peek >> (32 - kLutK - nb2)) & ((1u << nb2) - 1u));
    const uint32_t idx = s.esc ? l.base + sub : base2 + (peek2 >> (32 - kLutK));
    l.base = s.esc ? l.base : base2;
    l.e = lut[idx];
    l.p += total;
    return s;
}

// the part of the bookkeeping that is not needed to request the next entry
template <class Fetch>
JPGD_HD void step_finish(Lane& l, BitWin& w, const Step& s, const Syntax& sx, Fetch fetch) {
    l.nb += s.done ? 1u : 0u;
    if (s.done) {
        l.u4 = next_unit(l.u4, sx);
        set_unit(l, sx);
    }
    // without a branch: when no word was taken this re-reads the word already held
    w.next += s.need ? 1u : 0u;
    w.ahead = fetch(w.next);
}

// Synchronisation pass (write = false in Algorithm 2): decode while the next symbol starts before
// `limit`, keeping the state, the count of completed units and the per-component DC sums.
// The lane must have been primed.
template <class Fetch, class LutPtr>
JPGD_HD void decode_span_sync(Lane& l, BitWin& w, uint32_t limit, int64_t& dcacc, const Syntax& sx, Fetch fetch,
                              LutPtr lut) {
    while (l.p < limit) {
        const uint32_t comp = l.comp;
        const Step s = step_and_request(l, w, lut);
        const int32_t v = symbol_value(s.peek, s.len, s.size);
        const int32_t mul = s.is_dc ? (int32_t)(1u << (15u * comp)) : 0;
        dcacc += (int64_t)v * (int64_t)mul;
        step_finish(l, w, s, sx, fetch);
    }
}

// Write pass (write = true in Algorithm 2): the same walk, storing every non-zero coefficient at
// 64*unit + zig-zag index, DC values un-differenced.  `unit` is the index of the data unit being
// decoded, `total_units` the end of the image, pred0..2 the DC predictors; `flags` collects kSt* bits.
template <class Fetch, class LutPtr, class Store>
JPGD_HD void decode_span_write(Lane& l, BitWin& w, uint32_t limit, uint32_t& unit, uint32_t total_units,
                               int32_t& pred0, int32_t& pred1, int32_t& pred2, const Syntax& sx, Fetch fetch,
                               LutPtr lut, Store store, uint32_t& flags) {
    while (l.p < limit && unit < total_units) {
        const uint32_t comp = l.comp;
        const Step s = step_and_request(l, w, lut);
        const int32_t value = symbol_value(s.peek, s.len, s.size);
        if (!s.esc) {
            if (s.adv == 0u) flags |= kStInvalid;  // no codeword starts with these bits
            if (s.is_dc) {
                int32_t pred = comp == 0u ? pred0 : (comp == 1u ? pred1 : pred2);
                pred += value;
                pred0 = comp == 0u ? pred : pred0;
                pred1 = comp == 1u ? pred : pred1;
                pred2 = comp == 2u ? pred : pred2;
                if (s.adv) store(unit, 0u, (int16_t)pred);
            } else if (s.size) {
                const uint32_t at = s.z + s.adv - 1u;  // after the run of zeros
                if (at < 64u) store(unit, at, (int16_t)value);
                else flags |= kStInvalid;
            } else if (s.adv == 16u && s.z + 16u > 64u) {
                flags |= kStInvalid;  // ZRL running past the end of the unit
            }
        }
        if (s.done) unit++;
        step_finish(l, w, s, sx, fetch);
    }
}

}  // namespace jpgd
