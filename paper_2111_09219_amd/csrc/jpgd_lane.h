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

// What a lane needs to know about one data unit of the MCU: where the tables of its symbols are, which
// DC sum it feeds, and which unit follows.  One row per data unit, 16 bytes, read as a whole.
struct alignas(16) UnitRow {
    uint32_t tb_ac;       // first entry of the unit's AC table inside the LUT array
    uint32_t tb_dc_next;  // first entry of the DC table of the unit that follows
    uint32_t dcmul;       // 1 << (15 * component): the component's field of the packed DC sums
    uint32_t next;        // index of the unit that follows
};

// sched_*: 4 bits per data unit (see ImgDesc)
JPGD_HD UnitRow make_unit_row(uint32_t u, uint32_t upm, uint32_t sched_dc, uint32_t sched_ac, uint32_t sched_comp) {
    UnitRow r;
    const uint32_t un = u + 1u == upm ? 0u : u + 1u;
    r.tb_ac = ((sched_ac >> (4u * u)) & 15u) * (uint32_t)kLutEntries;
    r.tb_dc_next = ((sched_dc >> (4u * un)) & 15u) * (uint32_t)kLutEntries;
    r.dcmul = 1u << (15u * ((sched_comp >> (4u * u)) & 15u));
    r.next = un;
    return r;
}

// Decoder state of the paper, (p, n, c, z), with c refined to the data unit inside the MCU
// (two decoders inside different luminance units of a 4:2:0 MCU agree on the component but
// not on what follows) and n kept as completed data units (see SInfo).
struct Lane {
    uint32_t p;    // bit position in the unstuffed stream of the next syntax element (kept by the window inside the
                   // decode loops, written back when they end)
    uint32_t u;    // data unit inside the MCU
    uint32_t z;    // zig-zag index of the next coefficient (0 = a DC symbol is next)
    uint32_t nb;   // data units completed since the counter was last cleared
    // pipeline registers (prime)
    uint32_t e;    // table entry already read for the symbol at p (possibly a first-level escape)
    uint32_t base; // table that entry came from
    // synchronisation pass with two symbols per step (decode_span_sync_pairs)
    uint32_t pb;   // pair byte read for the symbol at p, as if that symbol came from unit u's AC table
};

// Window on the stream: two consecutive big-endian words and the offset of the next unread bit in the
// first; `peek` is the 32 bits that start there (a codeword has at most 16 bits, its value at most 16).
struct BitWin {
    uint32_t hi, lo;
    uint32_t o;      // 0..31
    uint32_t peek;
    uint32_t next;   // cursor of the word held in `ahead`, in the units of the Fetch functor; hi is word next - 2
    uint32_t ahead;  // the word after `lo`, fetched one refill early so that its latency is hidden
    uint32_t origin; // bit position in the stream of the word with cursor 0
};

// bit position of the next unread bit
JPGD_HD uint32_t win_pos(const BitWin& w) { return w.origin + ((w.next - 2u) << 5) + w.o; }
// the window has reached bit `limit` (a multiple of 32) as soon as its cursor `next` has reached this value
JPGD_HD uint32_t win_stop(const BitWin& w, uint32_t limit) { return ((limit - w.origin) >> 5) + 2u; }

// per-image constants of the scan syntax
struct Syntax {
    const UnitRow* rows;  // one per data unit of the MCU
    uint32_t upm;         // units per MCU
    const uint32_t* pair_of_unit = nullptr;  // per data unit: offset of its AC table's pair bytes (kernels that use them)
};

JPGD_HD uint32_t win_peek(const BitWin& w) {
    return (uint32_t)(((((uint64_t)w.hi << 32) | (uint64_t)w.lo) << w.o) >> 32);
}

// `cursor` addresses the 32-bit word that holds bit p
template <class Fetch>
JPGD_HD void win_init(BitWin& w, uint32_t p, uint32_t cursor, Fetch fetch) {
    w.hi = fetch(cursor);
    w.lo = fetch(cursor + 1u);
    w.o = p & 31u;
    w.peek = win_peek(w);
    w.next = cursor + 2u;
    w.ahead = fetch(w.next);
    w.origin = (p & ~31u) - (cursor << 5);
}

// Starts the pipeline: after (p, u, z) and the window are set, read the entry of the symbol at p.
template <class LutPtr>
JPGD_HD void prime(Lane& l, const BitWin& w, const Syntax& sx, LutPtr lut) {
    const uint32_t tb_dc = sx.rows[l.u == 0u ? sx.upm - 1u : l.u - 1u].tb_dc_next;
    l.base = l.z == 0u ? tb_dc : sx.rows[l.u].tb_ac;
    l.e = lut[l.base + (w.peek >> (32 - kLutK))];
}

// The value bits are the last `size` of the `total` bits a symbol takes; "signed ones' complement" (paper,
// Section 2): a leading 1 means the bits are the value itself, a leading 0 means value = bits - (2^size - 1);
// size 0 gives 0.  peek holds the symbol from its most significant bit on.  With the field read as a signed
// number s (leading 1 = negative): value = s + 2^size if s < 0, else s - 2^size + 1.
JPGD_HD int32_t symbol_value(uint32_t peek, uint32_t total, uint32_t size) {
#if defined(__HIP_DEVICE_COMPILE__)
    const int32_t s = __builtin_amdgcn_sbfe((int32_t)peek, (32u - total) & 31u, size);
#else
    const uint32_t raw = (peek >> ((32u - total) & 31u)) & ((1u << size) - 1u);
    const int32_t s = size ? (int32_t)(raw << (32u - size)) >> (32u - size) : 0;
#endif
    // s + 2^size if s < 0, s - (2^size - 1) otherwise: subtract 2^size - 1 with all its bits flipped in the first case
    return s - (int32_t)(((1u << size) - 1u) ^ (uint32_t)(s >> 31));
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
    uint32_t total, size, adv;  // bits taken, value bits among them, zig-zag slots covered
    bool esc;        // first-level escape: nothing was consumed, the state did not change
    bool is_dc;
    bool done;       // the symbol completed its data unit
    bool need;       // the window moved on by a word
    uint32_t z;      // zig-zag index the symbol started at
    uint32_t dcmul;  // of the data unit the symbol belongs to
};

// The row of the current unit is read at the top of the step and used at its end (which table the next entry comes
// from); the next stream word is asked for in the middle and used in the next step; the table entry is asked for
// last and is what the next step starts with.  Nothing but the entry and the window is carried from step to step
// in registers.
template <class Fetch, class LutPtr>
JPGD_HD Step step_and_request(Lane& l, BitWin& w, const Syntax& sx, Fetch fetch, LutPtr lut) {
    Step s;
    const UnitRow old = sx.rows[l.u];
    const uint32_t e = l.e;
    s.peek = w.peek;
    s.esc = lut_esc(e);
    const uint32_t ee = s.esc ? 0u : e;
    s.total = lut_total(ee);  // at most 31
    s.size = lut_size(ee);
    s.adv = lut_adv(ee);
    s.is_dc = l.z == 0u;
    s.z = l.z;
    const uint32_t o2 = w.o + s.total;
    s.need = o2 >= 32u;
    const uint32_t zn = l.z + s.adv;
    s.done = zn >= 64u;
    // off the chain, without branches: when no word is taken the word already held is read again, when the
    // unit does not change its row is
    w.next += s.need ? 1u : 0u;
    const uint32_t ahead = fetch(w.next);
    l.u = s.done ? old.next : l.u;
    s.dcmul = old.dcmul;
    l.nb += s.done ? 1u : 0u;
    // window past the symbol
    w.o = o2 & 31u;
    w.hi = s.need ? w.lo : w.hi;
    w.lo = s.need ? w.ahead : w.lo;
    w.ahead = ahead;
    w.peek = win_peek(w);
    l.z = s.done ? 0u : zn;
    // request: next symbol from the DC table of the next unit or the AC table of this one; an escape asks
    // the second level of the table it came from
    uint32_t base2 = s.done ? old.tb_dc_next : old.tb_ac;
#if defined(__HIP_DEVICE_COMPILE__)
    // (Only the arm for ordinary entries below uses base2, and the compiler would move the read of the row into that
    // arm and wait for it there; this keeps the read at the top of the step.)
    asm volatile("" : "+v"(base2));
#endif
    const uint32_t nb2 = lut_esc_bits(e);
    const uint32_t sub = (uint32_t)kLutL1 + lut_esc_offset(e) + ((s.peek >> (32 - kLutK - nb2)) & ((1u << nb2) - 1u));
    const uint32_t idx = s.esc ? l.base + sub : base2 + (w.peek >> (32 - kLutK));
    l.base = s.esc ? l.base : base2;
    l.e = lut[idx];
    return s;
}

// One symbol of the synchronisation pass (write = false in Algorithm 2): state, count of completed units
// (inside step_and_request) and the per-component sums of DC differences.
template <class Fetch, class LutPtr>
JPGD_HD void sync_symbol(Lane& l, BitWin& w, int64_t& dcacc, const Syntax& sx, Fetch fetch, LutPtr lut) {
    const Step s = step_and_request(l, w, sx, fetch, lut);
    const int32_t v = symbol_value(s.peek, s.total, s.size);
    const int32_t mul = s.is_dc ? (int32_t)s.dcmul : 0;
    dcacc += (int64_t)v * (int64_t)mul;
}

// Synchronisation pass: decode while the next symbol starts before `limit`.  The lane must have been primed.
template <class Fetch, class LutPtr>
JPGD_HD void decode_span_sync(Lane& l, BitWin& w, uint32_t limit, int64_t& dcacc, const Syntax& sx, Fetch fetch,
                              LutPtr lut) {
    const uint32_t stop = win_stop(w, limit);
    while (w.next < stop) sync_symbol(l, w, dcacc, sx, fetch, lut);
    l.p = win_pos(w);
}

// ---- two symbols per step ---------------------------------------------------------------------------------
// The synchronisation pass needs the state, the unit count and the DC sums, not the coefficients.  So where the
// first-level index of an AC symbol also holds the whole codeword of the AC symbol after it, one step may take
// both: the pair byte of that index (build_pairs) says how many bits the second symbol takes and how many slots it
// covers.  The second symbol is taken only if the first one is an AC symbol that leaves its data unit open (the
// second then belongs to the same unit and the same table); the step is exactly two steps of sync_symbol.
template <class Fetch, class LutPtr, class PairPtr>
JPGD_HD void sync_symbol_pair(Lane& l, BitWin& w, int64_t& dcacc, const Syntax& sx, Fetch fetch, LutPtr lut,
                              PairPtr pairs) {
    const UnitRow row = sx.rows[l.u];
    const uint32_t pair = sx.pair_of_unit[l.u];
    const uint32_t e = l.e;
    const uint32_t peek = w.peek;
    const bool esc = lut_esc(e);
    const uint32_t ee = esc ? 0u : e;
    const uint32_t t1 = lut_total(ee), size = lut_size(ee), a1 = lut_adv(ee);
    const bool is_dc = l.z == 0u;
    const uint32_t zn1 = l.z + a1;
    const uint32_t pb = (is_dc || zn1 >= 64u) ? 0u : l.pb;  // (an escape's index has pair byte 0)
    const uint32_t a2c = pb >> 4;
    const uint32_t total = t1 + (pb & 15u);
    const uint32_t zn = zn1 + a2c;
    const bool done = zn >= 64u || a2c == 15u;  // 15: the second symbol is end-of-block
    const uint32_t o2 = w.o + total;  // at most 31 + 20 + 15
    const bool need = o2 >= 32u;
    w.next += need ? 1u : 0u;
    const uint32_t ahead = fetch(w.next);
    l.nb += done ? 1u : 0u;
    w.o = o2 & 31u;
    w.hi = need ? w.lo : w.hi;
    w.lo = need ? w.ahead : w.lo;
    w.ahead = ahead;
    w.peek = win_peek(w);
    l.z = done ? 0u : zn;
    l.u = done ? row.next : l.u;
    uint32_t base2 = done ? row.tb_dc_next : row.tb_ac;
#if defined(__HIP_DEVICE_COMPILE__)
    // (Only the arm for ordinary entries below uses base2, and the compiler would move the read of the row into that
    // arm and wait for it there; this keeps the read at the top of the step.)
    asm volatile("" : "+v"(base2));
#endif
    const uint32_t nb2 = lut_esc_bits(e);
    const uint32_t sub = (uint32_t)kLutL1 + lut_esc_offset(e) + ((peek >> (32 - kLutK - nb2)) & ((1u << nb2) - 1u));
    const uint32_t i1 = w.peek >> (32 - kLutK);
    const uint32_t idx = esc ? l.base + sub : base2 + i1;
    l.base = esc ? l.base : base2;
    l.e = lut[idx];
    // asked as if the next symbol came from the AC table of the unit just left: if the unit is complete the next
    // symbol is a DC symbol and the byte is not looked at
    l.pb = pairs[pair + i1];
    const int32_t v = symbol_value(peek, t1, size);
    dcacc += (int64_t)v * (int64_t)(is_dc ? (int32_t)row.dcmul : 0);
}

// The synchronisation pass with pairs.  A second symbol must start before `limit` like any other: pairs are taken
// while the step starts at least 32 bits before it (a first symbol with a pair byte has at most 20 bits), single
// symbols from there on.  The lane must have been primed; sx.pair_of_unit must be set.
template <class Fetch, class LutPtr, class PairPtr>
JPGD_HD void decode_span_sync_pairs(Lane& l, BitWin& w, uint32_t limit, int64_t& dcacc, const Syntax& sx, Fetch fetch,
                                    LutPtr lut, PairPtr pairs) {
    const uint32_t stop = win_stop(w, limit);
    l.pb = pairs[sx.pair_of_unit[l.u] + (w.peek >> (32 - kLutK))];
#if defined(__HIP_DEVICE_COMPILE__)
    // (Keeps the compiler from merging this read with the one at the end of a step into a single read at the top of
    // the loop, where every step would wait for it: the byte is asked for one step ahead, like the table entry.)
    asm volatile("" : "+v"(l.pb));
#endif
    while (w.next + 1u < stop) sync_symbol_pair(l, w, dcacc, sx, fetch, lut, pairs);
    while (w.next < stop) sync_symbol(l, w, dcacc, sx, fetch, lut);
    l.p = win_pos(w);
}

// One symbol of the write pass (write = true in Algorithm 2): every non-zero coefficient goes to
// 64*unit + zig-zag index, DC values un-differenced.  `unit` is the index of the data unit being decoded,
// pred0..2 the DC predictors; `flags` collects kSt* bits.  Without branches except around the store itself:
// a wavefront holds lanes in every kind of symbol at once, so each arm of a branch would be walked anyway.
template <class Fetch, class LutPtr, class Store>
JPGD_HD void write_symbol(Lane& l, BitWin& w, uint32_t& unit, int32_t& pred0, int32_t& pred1, int32_t& pred2,
                          const Syntax& sx, Fetch fetch, LutPtr lut, Store store, uint32_t& flags) {
    const Step s = step_and_request(l, w, sx, fetch, lut);
    const bool comp0 = s.dcmul == 1u, comp1 = s.dcmul == (1u << 15);
    const int32_t value = symbol_value(s.peek, s.total, s.size);  // 0 for an escape
    const bool real = !s.esc;
    const bool dc = s.is_dc && real;
    const int32_t pred = (comp0 ? pred0 : (comp1 ? pred1 : pred2)) + value;
    pred0 = dc && comp0 ? pred : pred0;
    pred1 = dc && comp1 ? pred : pred1;
    pred2 = dc && !comp0 && !comp1 ? pred : pred2;
    // where the symbol ends: a coefficient sits in the last slot it covers (after its run of zeros)
    const uint32_t zn = s.z + s.adv;
    const uint32_t at = dc ? 0u : zn - 1u;
    const bool has_value = dc || s.size != 0u;  // a DC symbol of size 0 still yields the predictor
    if (real && s.adv != 0u && has_value && at < 64u) store(unit, at, (int16_t)(dc ? pred : value));
    // no codeword starts with these bits; or a coefficient or a run of sixteen zeros (not end-of-block,
    // which may be coded anywhere) that runs past the end of the unit
    const bool bad = real && (s.adv == 0u || (zn > 64u && s.adv != kAdvEob));
    flags |= bad ? kStInvalid : 0u;
    unit += s.done ? 1u : 0u;
}

// Write pass: the same walk as the synchronisation pass, up to the image's last data unit.
template <class Fetch, class LutPtr, class Store>
JPGD_HD void decode_span_write(Lane& l, BitWin& w, uint32_t limit, uint32_t& unit, uint32_t total_units,
                               int32_t& pred0, int32_t& pred1, int32_t& pred2, const Syntax& sx, Fetch fetch,
                               LutPtr lut, Store store, uint32_t& flags) {
    const uint32_t stop = win_stop(w, limit);
    while (w.next < stop && unit < total_units) write_symbol(l, w, unit, pred0, pred1, pred2, sx, fetch, lut, store, flags);
    l.p = win_pos(w);
}

// ---- restart intervals -------------------------------------------------------------------------------
// A scan with restart intervals (DRI) is a chain of independently coded intervals: each ends with up to seven
// 1-bits of padding and a marker RSTm, and the next starts byte-aligned with the DC predictors at zero.  The
// unstuff kernels drop the markers and mark the first byte of every interval in a bitmap (one bit per byte
// of the unstuffed stream; bit b of word k stands for byte 32k + b).  The paper does not treat restart
// markers.  The rules below are stated on positions alone, so that a decoder in any state obeys them, and on
// the synchronised chain they are what a sequential decoder does:
//   * after a symbol, if the next interval starts at most 7 bits further on and those bits are all 1, or if
//     the symbol ran past that start, the decoder moves to the start with z = 0 and u = 0 (a real symbol
//     never consists of 1-bits only: the all-ones codeword is reserved);
//   * a symbol that starts at the first bit of an interval finds the DC sums / predictors at zero.
// Every decoder is therefore synchronised from the next interval on, whatever it did before.

constexpr uint32_t kNoBoundary = 0xFFFFFFFFu;

// first bit position B >= from_bit, B < end_bit, at which an interval starts; bword(k) = word k of the bitmap
template <class BWord>
JPGD_HD uint32_t next_boundary(uint32_t from_bit, uint32_t end_bit, BWord bword) {
    const uint32_t byte = (from_bit + 7u) >> 3, endb = (end_bit + 7u) >> 3;
    if (byte >= endb) return kNoBoundary;
    uint32_t k = byte >> 5;
    uint32_t m = bword(k) & (0xFFFFFFFFu << (byte & 31u));
    for (;;) {
        if (m) {
            const uint32_t b = (k << 5) + (uint32_t)__builtin_ctz(m);
            return b < endb ? b << 3 : kNoBoundary;
        }
        ++k;
        if ((k << 5) >= endb) return kNoBoundary;
        m = bword(k);
    }
}

// the window moves to bit B (a multiple of 8) and the decoder starts a fresh MCU there
template <class Fetch, class LutPtr>
JPGD_HD void move_to_interval(Lane& l, BitWin& w, uint32_t B, const Syntax& sx, Fetch fetch, LutPtr lut) {
    l.z = 0u;
    l.u = 0u;
    win_init(w, B, (B - w.origin) >> 5, fetch);
    prime(l, w, sx, lut);
}

// after a symbol: has the decoder reached the padding in front of the interval that starts at B, or passed B?
JPGD_HD bool at_interval_end(const BitWin& w, uint32_t pos, uint32_t B) {
    if (pos >= B) return true;
    const uint32_t r = B - pos;
    return r <= 7u && (~w.peek >> (32u - r)) == 0u;
}

// Where the fast part of a span ends when the next interval starts at B: a symbol that starts before `calm` ends more
// than 7 bits before B (it has at most 31 bits), so nothing has to be checked on the way there.  As a window cursor.
JPGD_HD uint32_t calm_stop(const BitWin& w, uint32_t B, uint32_t limit) {
    uint32_t calm = limit;
    if (B != kNoBoundary) {
        const uint32_t c = B >= 40u ? (B - 39u) & ~31u : 0u;
        calm = c < limit ? c : limit;
    }
    return calm > w.origin ? win_stop(w, calm) : 0u;
}

// Synchronisation pass over a stream with restart intervals.  `crossed` is set when a symbol of this span
// started an interval (dcacc then holds the sums since the last such symbol).
// A fast loop up to the neighbourhood of the next interval start, then a careful loop.  (The single loop of the
// write pass below was measured here too: the overflow rounds are a chain of dependent symbols in a lone
// wavefront, and the extra tests per symbol cost them more -- 4096x4096 with one interval per MCU row: 0.93
// against 0.78 ms -- than walking a span twice costs the few wavefronts that meet an interval start.)
template <class Fetch, class LutPtr, class BWord>
JPGD_HD void decode_span_sync_rst(Lane& l, BitWin& w, uint32_t limit, int64_t& dcacc, uint32_t& crossed, const Syntax& sx,
                                  Fetch fetch, LutPtr lut, BWord bword) {
    uint32_t from = win_pos(w);
    for (;;) {
        const uint32_t B = next_boundary(from, limit + 64u, bword);
        const uint32_t stop = calm_stop(w, B, limit);
        while (w.next < stop) sync_symbol(l, w, dcacc, sx, fetch, lut);
        if (B == kNoBoundary) break;
        uint32_t pos = win_pos(w);
        bool next_interval = false;
        while (pos < limit) {
            if (pos == B) {  // this symbol starts the interval
                dcacc = 0;
                crossed = 1u;
                from = B + 1u;
                next_interval = true;
                break;
            }
            sync_symbol(l, w, dcacc, sx, fetch, lut);
            pos = win_pos(w);
            if (at_interval_end(w, pos, B)) {
                move_to_interval(l, w, B, sx, fetch, lut);
                pos = B;
            }
        }
        if (!next_interval) break;
    }
    l.p = win_pos(w);
}

// Write pass over a stream with restart intervals: the predictors return to zero where an interval starts.
// An interval holds units_per_interval data units (all but the last of the scan): a start reached at any
// other unit count means damaged data and is flagged.
// One loop for all lanes: a lane near an interval start does its checks before and after the same write_symbol the
// others execute.  With a fast loop and a careful loop one after the other, a wavefront in which a few lanes meet
// an interval start walks its span up to three times (the fast loop for the others, the careful one, the fast
// one again for what follows the start); the write kernel, whose wavefronts all have full spans to decode, is a
// third faster this way on streams with one interval per MCU row.
template <class Fetch, class LutPtr, class Store, class BWord>
JPGD_HD void decode_span_write_rst(Lane& l, BitWin& w, uint32_t limit, uint32_t& unit, uint32_t total_units,
                                   uint32_t units_per_interval, int32_t& pred0, int32_t& pred1, int32_t& pred2,
                                   const Syntax& sx, Fetch fetch, LutPtr lut, Store store, uint32_t& flags, BWord bword) {
    uint32_t B = next_boundary(win_pos(w), limit + 64u, bword);
    uint32_t stop = calm_stop(w, B, limit);
    while (unit < total_units) {
        const bool near = w.next >= stop;
        if (near) {
            if (B == kNoBoundary) break;
            const uint32_t pos = win_pos(w);
            if (pos >= limit) break;
            if (pos == B) {
                pred0 = pred1 = pred2 = 0;
                if (unit % units_per_interval != 0u) flags |= kStInvalid;
                B = next_boundary(B + 1u, limit + 64u, bword);
                stop = calm_stop(w, B, limit);
                continue;
            }
        }
        write_symbol(l, w, unit, pred0, pred1, pred2, sx, fetch, lut, store, flags);
        if (near && at_interval_end(w, win_pos(w), B)) move_to_interval(l, w, B, sx, fetch, lut);
    }
    l.p = win_pos(w);
}

}  // namespace jpgd
