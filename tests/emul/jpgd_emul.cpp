// Host walk-through of the decoder's kernels: the same lane code (jpgd_lane.h, jpgd_lut.h, jpgd_idct.h)
// and the same index arithmetic as jpgd_kernels.h, with workgroups and lanes run one after another.
// It exists so that the CPU-only test run can check the host logic (tables, lane decoder, record
// packing, padded staging layout, scan, write, pixel arithmetic) before anything reaches a GPU.
// It is test code: the library never calls it and it is not a fallback for the GPU path.
//
// Build: g++ -O2 -std=c++17 -shared -fPIC -o libjpgd_emul.so jpgd_emul.cpp ../../paper_2111_09219_amd/csrc/jpgd_parse.cpp
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "../../include/jpgd.h"
#include "../../paper_2111_09219_amd/csrc/jpgd_common.h"
#include "../../paper_2111_09219_amd/csrc/jpgd_idct.h"
#include "../../paper_2111_09219_amd/csrc/jpgd_lane.h"
#include "../../paper_2111_09219_amd/csrc/jpgd_lut.h"

using namespace jpgd;

namespace {

uint32_t bswap(uint32_t v) { return __builtin_bswap32(v); }
int32_t sx16(uint32_t v) { return (int32_t)(int16_t)(v & 0xFFFFu); }
uint32_t pack_dc01(int64_t acc) { int32_t a, b, c; dc_unpack(acc, a, b, c); return ((uint32_t)a & 0xFFFFu) | ((uint32_t)b << 16); }
uint32_t pack_dc2(int64_t acc) { int32_t a, b, c; dc_unpack(acc, a, b, c); return (uint32_t)c & 0xFFFFu; }

struct Image {
    jpgd_info in;
    uint32_t sched_dc = 0, sched_ac = 0, sched_comp = 0, nslots = 0;
    std::vector<uint16_t> lut;
    std::vector<uint8_t> pairs;    // pair bytes of the AC tables, AC table k at k * kPairBytes
    uint32_t pair_of_unit[8] = {0};
    std::vector<uint8_t> stream;  // unstuffed + zero slack
    std::vector<uint32_t> bmap;   // restart intervals: one bit per unstuffed byte, set at the first byte of an interval
    uint32_t nbytes = 0, nsub = 0, markers = 0;
};

int prepare(const uint8_t* file, size_t len, Image& im) {
    int rc = jpgd_parse(file, len, &im.in);
    if (rc) return rc;
    const jpgd_info& in = im.in;
    uint32_t dc_ids[3], ac_ids[3], ndc = 0, nac = 0, cdc[3], cac[3];
    for (uint32_t c = 0; c < in.ncomp; ++c) {
        uint32_t k;
        for (k = 0; k < ndc && dc_ids[k] != in.td[c]; ++k) {}
        if (k == ndc) dc_ids[ndc++] = in.td[c];
        cdc[c] = k;
        for (k = 0; k < nac && ac_ids[k] != in.ta[c]; ++k) {}
        if (k == nac) ac_ids[nac++] = in.ta[c];
        cac[c] = k;
    }
    im.nslots = ndc + nac;
    im.lut.assign((size_t)im.nslots * kLutEntries, 0);
    im.pairs.assign((size_t)nac * kPairBytes, 0);
    uint32_t u = 0;
    for (uint32_t c = 0; c < in.ncomp; ++c) {
        uint32_t nu = (in.ncomp == 1) ? 1u : (c == 0 ? (uint32_t)in.hsamp[0] * in.vsamp[0] : 1u);
        for (uint32_t k = 0; k < nu; ++k, ++u) {
            im.sched_dc |= cdc[c] << (4 * u);
            im.sched_ac |= (ndc + cac[c]) << (4 * u);
            im.sched_comp |= c << (4 * u);
            im.pair_of_unit[u] = cac[c] * (uint32_t)kPairBytes;
        }
        if (!build_lut(in.dht_bits[0][in.td[c]], in.dht_vals[0][in.td[c]], true, &im.lut[(size_t)cdc[c] * kLutEntries]) ||
            !build_lut(in.dht_bits[1][in.ta[c]], in.dht_vals[1][in.ta[c]], false, &im.lut[(size_t)(ndc + cac[c]) * kLutEntries]))
            return JPGD_E_TABLE;
        build_pairs(&im.lut[(size_t)(ndc + cac[c]) * kLutEntries], &im.pairs[(size_t)cac[c] * kPairBytes]);
    }
    return JPGD_OK;
}

// the two unstuff kernels, tile by tile and lane by lane
void unstuff(const uint8_t* scan, uint32_t n, uint32_t logL, Image& im) {
    const uint32_t tiles = (n + kUnstuffTile - 1) / kUnstuffTile;
    const bool restart = im.in.restart_interval != 0;
    std::vector<uint32_t> removed(tiles, 0), before(tiles, 0);
    auto keep_mask = [&](uint32_t pos, uint32_t& nvalid, uint32_t& marks) {
        nvalid = pos >= n ? 0u : std::min(16u, n - pos);
        uint32_t prev = (pos > 0 && nvalid) ? scan[pos - 1] : 0u, mask = 0;
        marks = 0;
        for (uint32_t j = 0; j < nvalid; ++j) {
            uint32_t b = scan[pos + j];
            bool nx_exists = pos + j + 1 < n;
            uint32_t nx = nx_exists ? scan[pos + j + 1] : 0u;
            bool rst2 = restart && prev == 255 && (b & 0xF8) == 0xD0;
            bool rst1 = restart && b == 255 && nx_exists && (nx & 0xF8) == 0xD0;
            if (!((b == 0 && prev == 255) || rst1 || rst2)) mask |= 1u << j;
            if (rst2) marks |= 1u << j;
            prev = b;
        }
        return mask;
    };
    im.markers = 0;
    for (uint32_t t = 0; t < tiles; ++t)
        for (uint32_t lane = 0; lane < (uint32_t)kWG; ++lane) {
            uint32_t nv, mk, m = keep_mask(t * kUnstuffTile + lane * 16, nv, mk);
            removed[t] += nv - (uint32_t)__builtin_popcount(m);
            im.markers += (uint32_t)__builtin_popcount(mk);
        }
    uint32_t carry = 0;
    for (uint32_t t = 0; t < tiles; ++t) { before[t] = carry; carry += removed[t]; }
    im.nbytes = n - carry;
    const uint32_t L = 1u << logL;
    im.nsub = (uint32_t)(((uint64_t)im.nbytes * 8 + L - 1) >> logL);
    im.stream.assign((size_t)n + L / 8 + 64 + 16 + 256, 0xAA);  // poison: the kernels must define what they read
    im.bmap.assign((size_t)tiles * 128 + 128, 0);
    for (uint32_t t = 0; t < tiles; ++t) {
        uint32_t o = t * kUnstuffTile - before[t];
        for (uint32_t lane = 0; lane < (uint32_t)kWG; ++lane) {
            uint32_t pos = t * kUnstuffTile + lane * 16, nv, mk, m = keep_mask(pos, nv, mk);
            for (uint32_t j = 0; j < nv; ++j) {
                if (mk & (1u << j)) im.bmap[o >> 5] |= 1u << (o & 31);  // the next kept byte starts an interval
                if (m & (1u << j)) im.stream[o++] = scan[pos + j];
            }
        }
    }
    for (uint32_t k = 0; k < L / 8 + 64; ++k) im.stream[im.nbytes + k] = 0;
}

struct Emul {
    Image im;
    uint32_t logL, H, seq_len;
    std::vector<SInfo> sinfo;
    std::vector<uint32_t> warm;  // per sequence: the state its records continue (0xFFFFFFFF = none)
    UnitRow rows[8];
    Syntax sx;
    uint32_t inter_changed = 0, rounds_max = 0, flags = 0, pending = 0;
};

// The wavefront-per-chain decoder of jpgd_kernels.h (coop_unit_word, coop_span_sync) with its 64 lanes run
// one after another: the same table words, the same 64-word stretch held by the lanes, the same four answers
// per lane, the same grid of windows and the same walk through them (the kernel asks for the next window's
// answers ahead of time and follows up the escapes of all lanes at the first one the chain meets; here each is
// followed up when the chain meets it, which gives the same entries).
uint32_t g_coop_max = kCoopMax;  // as the library sets it for four wavefronts; the tests also run with 0 (never), 8 and 64
uint32_t g_sync_waves = kWG / 64;  // wavefronts per workgroup (the library launches 4, 8 or 16)

uint32_t coop_unit_word(const Syntax& sx, uint32_t lane) {
    if (lane >= sx.upm) return 0u;
    const UnitRow r = sx.rows[lane];
    return (r.tb_ac / (uint32_t)kLutEntries) | ((r.tb_dc_next / (uint32_t)kLutEntries) << 3) | (r.next << 6) |
           (((uint32_t)__builtin_ffs((int)r.dcmul) - 1u) << 10);
}

uint32_t coop_resolve(const uint16_t* lut, uint32_t slot, uint32_t e, uint32_t peek) {
    const uint32_t nb2 = lut_esc_bits(e);
    return lut[slot * (uint32_t)kLutEntries + (uint32_t)kLutL1 + lut_esc_offset(e) +
               ((peek >> (32 - kLutK - nb2)) & ((1u << nb2) - 1u))];
}

uint32_t coop_step(uint32_t e) { return (e & 0x8000u) ? 0x10000u : ((e & 0x7E00u) | std::max(e & 31u, 1u)); }

template <class Fetch>
void coop_span_sync(uint32_t& p, uint32_t& u, uint32_t& z, uint32_t& nb, int64_t& dc, uint32_t limit, uint32_t org_word,
                    uint32_t nwords, const uint32_t unit_word[64], uint32_t upm, uint32_t nslots, Fetch fetch,
                    const uint16_t* lut) {
    nb = 0;
    dc = 0;
    uint32_t cur = unit_word[u];
    uint32_t ac_slot = cur & 7u;
    uint32_t dc_slot = (unit_word[u == 0u ? upm - 1u : u - 1u] >> 3) & 7u;
    uint32_t w0 = 0, held[64];
    bool have = false;
    if (p >= limit) return;
    // windows of 64 bit positions on a 64-bit grid of the stream (a subsequence is a whole number of them); the
    // chain enters a window where the last symbol of the window before ended
    uint32_t ws = p & ~63u;
    uint32_t S = (p - ws) | (z << 9);
    for (;; ws += 64u) {
        uint32_t wb = (ws >> 5) - w0;
        if (!have || wb + 2u > 63u) {
            w0 = ws >> 5;
            for (uint32_t lane = 0; lane < 64; ++lane) {
                const uint32_t c = w0 - org_word + lane;
                held[lane] = c < nwords ? fetch(c) : 0u;
            }
            wb = 0;
            have = true;
        }
        uint32_t peek[64], e01[64], e23[64];
        for (uint32_t lane = 0; lane < 64; ++lane) {
            const uint32_t off = lane >> 5;
            const uint32_t hi = held[wb + off], lo = held[wb + off + 1u];
            peek[lane] = (uint32_t)(((((uint64_t)hi << 32) | (uint64_t)lo) << (lane & 31u)) >> 32);
            const uint32_t idx = peek[lane] >> (32 - kLutK);
            uint32_t e[4];
            for (uint32_t s = 0; s < 4u; ++s) e[s] = lut[std::min(s, nslots - 1u) * (uint32_t)kLutEntries + idx];
            e01[lane] = e[0] | (e[1] << 16);
            e23[lane] = e[2] | (e[3] << 16);
        }
        auto entry = [&](uint32_t slot, uint32_t j) { return ((slot & 2u) ? e23[j] : e01[j]) >> ((slot & 1u) << 4); };
        if ((S & 0x7Fu) >= 64u) abort();  // a symbol has at most 31 bits: the chain enters within the window
        for (;;) {
            if ((S >> 9) == 0u) {
                uint32_t r = entry(dc_slot, S);
                if (r & 0x8000u) r = coop_resolve(lut, dc_slot, r, peek[S]);
                dc += (int64_t)symbol_value(peek[S], lut_total(r), lut_size(r)) * (int64_t)(1u << ((cur >> 10) & 31u));
                S += coop_step(r);
                if (S & 0x40u) break;
                if ((S >> 9) == 0u) continue;
            }
            for (;;) {
                S += coop_step(entry(ac_slot, S & 63u));
                if ((S & 0x18040u) == 0u) continue;
                if (S & 0x10000u) {
                    S &= 0xFFFFu;
                    const uint32_t j = S & 63u;
                    S += coop_step(coop_resolve(lut, ac_slot, entry(ac_slot, j), peek[j]));
                    if ((S & 0x8040u) == 0u) continue;
                }
                break;
            }
            if (S & 0x8000u) {
                ++nb;
                S &= 0x7Fu;
                u = (cur >> 6) & 15u;
                dc_slot = (cur >> 3) & 7u;
                cur = unit_word[u];
                ac_slot = cur & 7u;
            }
            if (S & 0x40u) break;
        }
        if (ws + 64u >= limit) break;
        S -= 64u;  // the same position, seen from the next window
    }
    p = ws + (S & 0x7Fu);
    z = S >> 9;
}

void sync_intra(Emul& E) {
    const Image& im = E.im;
    const uint32_t nsub = im.nsub, logL = E.logL, L = 1u << logL, wps = L >> 5;
    const uint32_t nseq = (nsub + E.seq_len - 1) / E.seq_len;
    const uint32_t* words = (const uint32_t*)im.stream.data();
    std::vector<uint32_t> strm;
    for (uint32_t wg = 0; wg < nseq; ++wg) {
        const int32_t base = (int32_t)(wg * E.seq_len) - (int32_t)E.H;
        const uint32_t first = base < 0 ? 0u : (uint32_t)base;
        const uint32_t t0 = (uint32_t)((int32_t)first - base);
        const uint32_t t1 = std::min<uint32_t>(kWG, (uint32_t)((int32_t)nsub - base));
        const uint32_t first_word = first * wps, nwords = (t1 - t0) * wps + 4;
        strm.assign(nwords, 0xDEADBEEF);
        for (uint32_t r = 0; r < nwords; ++r) strm[r] = bswap(words[first_word + r]);
        auto fetch = [&](uint32_t c) {
            if (c >= nwords) abort();  // a lane read outside the staged window
            return strm[c];
        };
        // the part of the bitmap the kernel stages with these words
        const bool restart = im.in.restart_interval != 0;
        const uint32_t bm_k0 = first_word >> 3, bm_n = ((first_word + nwords + 7) >> 3) - bm_k0 + 1;
        auto bword = [&](uint32_t k) {
            if (k < bm_k0 || k - bm_k0 >= bm_n) abort();  // a lane looked outside the staged bitmap
            return im.bmap[k];
        };
        uint32_t sw[kWG], pnb[kWG], pdc01[kWG], pdc2[kWG];
        Lane l[kWG];
        BitWin bw[kWG];
        int64_t dcacc[kWG];
        bool active[kWG];
        uint32_t tt[kWG];
        for (uint32_t t = 0; t < (uint32_t)kWG; ++t) {
            active[t] = false;
            if (t < t0 || t >= t1) continue;
            uint32_t i = (uint32_t)(base + (int32_t)t);
            l[t].p = i << logL; l[t].u = 0; l[t].z = 0; l[t].nb = 0;
            dcacc[t] = 0;
            win_init(bw[t], l[t].p, (l[t].p >> 5) - first_word, fetch);
            prime(l[t], bw[t], E.sx, im.lut.data());
            uint32_t limit = (i + 1) << logL;
            uint32_t crossed = 0;
            if (restart) decode_span_sync_rst(l[t], bw[t], limit, dcacc[t], crossed, E.sx, fetch, im.lut.data(), bword);
            else decode_span_sync_pairs(l[t], bw[t], limit, dcacc[t], E.sx, fetch, im.lut.data(), im.pairs.data());
            sw[t] = pack_state(l[t].p - limit, l[t].z, l[t].u);
            pnb[t] = l[t].nb | (crossed << 31);
            pdc01[t] = pack_dc01(dcacc[t]);
            pdc2[t] = pack_dc2(dcacc[t]);
            active[t] = t + 1 < t1;
            tt[t] = t + 1;
        }
        uint32_t rounds = 0;
        for (;;) {
            bool any = false;
            for (uint32_t t = 0; t < (uint32_t)kWG; ++t) any = any || active[t];
            if (!any) break;
            ++rounds;
            uint32_t now = 0;
            for (uint32_t t = 0; t < (uint32_t)kWG; ++t) now += active[t] ? 1u : 0u;
            const bool coop = im.nslots <= 4u && now <= (restart ? std::min(g_coop_max, g_sync_waves) : g_coop_max);  // stays true once it is
            uint32_t unit_word[64];
            for (uint32_t lane = 0; lane < 64; ++lane) unit_word[lane] = coop_unit_word(E.sx, lane);
            for (uint32_t t = 0; t < (uint32_t)kWG; ++t) {
                if (!active[t]) continue;
                if (coop) {
                    const uint32_t limit = ((uint32_t)(base + (int32_t)tt[t]) + 1) << logL;
                    uint32_t nb, crossed = 0;
                    // a chain whose stretch holds an interval start is decoded by one lane with the interval rules
                    if (!restart || next_boundary(l[t].p, limit + 64u, bword) == kNoBoundary) {
                        coop_span_sync(l[t].p, l[t].u, l[t].z, nb, dcacc[t], limit, first_word, nwords, unit_word, E.sx.upm,
                                       im.nslots, fetch, im.lut.data());
                    } else {
                        l[t].nb = 0;
                        dcacc[t] = 0;
                        win_init(bw[t], l[t].p, (l[t].p >> 5) - first_word, fetch);
                        prime(l[t], bw[t], E.sx, im.lut.data());
                        decode_span_sync_rst(l[t], bw[t], limit, dcacc[t], crossed, E.sx, fetch, im.lut.data(), bword);
                        nb = l[t].nb;
                    }
                    uint32_t x = pack_state(l[t].p - limit, l[t].z, l[t].u);
                    bool synced = x == sw[tt[t]];
                    sw[tt[t]] = x; pnb[tt[t]] = nb | (crossed << 31);
                    pdc01[tt[t]] = pack_dc01(dcacc[t]);
                    pdc2[tt[t]] = pack_dc2(dcacc[t]);
                    ++tt[t];
                    active[t] = !synced && tt[t] < t1;
                    continue;
                }
                l[t].nb = 0;
                dcacc[t] = 0;
                win_init(bw[t], l[t].p, (l[t].p >> 5) - first_word, fetch);  // a chain moved to another lane restarts its window
                prime(l[t], bw[t], E.sx, im.lut.data());
                uint32_t limit = ((uint32_t)(base + (int32_t)tt[t]) + 1) << logL;
                uint32_t crossed = 0;
                if (restart) decode_span_sync_rst(l[t], bw[t], limit, dcacc[t], crossed, E.sx, fetch, im.lut.data(), bword);
                else decode_span_sync_pairs(l[t], bw[t], limit, dcacc[t], E.sx, fetch, im.lut.data(), im.pairs.data());
                uint32_t x = pack_state(l[t].p - limit, l[t].z, l[t].u);
                bool synced = x == sw[tt[t]];
                sw[tt[t]] = x; pnb[tt[t]] = l[t].nb | (crossed << 31);
                pdc01[tt[t]] = pack_dc01(dcacc[t]);
                pdc2[tt[t]] = pack_dc2(dcacc[t]);
                ++tt[t];
                active[t] = !synced && tt[t] < t1;
            }
        }
        E.rounds_max = std::max(E.rounds_max, rounds);
        E.warm[wg] = (E.H > 0 && E.H - 1 >= t0) ? sw[E.H - 1] : 0xFFFFFFFFu;
        for (uint32_t t = std::max(t0, E.H); t < t1; ++t) {
            SInfo r = {sw[t], pnb[t], pdc01[t], pdc2[t]};
            E.sinfo[(uint32_t)(base + (int32_t)t)] = r;
        }
    }
}

void sync_inter(Emul& E) {
    const Image& im = E.im;
    const uint32_t nsub = im.nsub, logL = E.logL;
    const uint32_t* words = (const uint32_t*)im.stream.data();
    auto fetch = [&](uint32_t w) { return bswap(words[w]); };
    auto bword = [&](uint32_t k) { return im.bmap[k]; };
    const bool restart = im.in.restart_interval != 0;
    E.inter_changed = 0;
    // On the GPU all boundaries are looked at together: every lane reads the last record of the sequence before
    // its boundary when the kernel starts, whatever another lane does to that record later in the same round.
    std::vector<uint32_t> seen;
    for (uint32_t b = 0; (uint64_t)(b + 1) * E.seq_len < nsub; ++b) seen.push_back(E.sinfo[(b + 1) * E.seq_len - 1].x);
    for (uint32_t b = 0;; ++b) {
        uint64_t gfirst = (uint64_t)(b + 1) * E.seq_len;
        if (gfirst >= nsub) break;
        uint32_t g = (uint32_t)gfirst, gend = std::min(nsub, g + E.seq_len);
        uint32_t x0 = seen[b];
        if (E.warm[b + 1] == x0) continue;  // the two sequences already form one chain
        Lane l;
        BitWin w;
        l.p = (g << logL) + state_prel(x0); l.z = state_z(x0); l.u = state_u(x0);
        win_init(w, l.p, l.p >> 5, fetch);
        prime(l, w, E.sx, im.lut.data());
        bool first = true;
        for (;;) {
            l.nb = 0;
            int64_t dcacc = 0;
            uint32_t limit = (g + 1) << logL;
            uint32_t crossed = 0;
            if (restart) decode_span_sync_rst(l, w, limit, dcacc, crossed, E.sx, fetch, im.lut.data(), bword);
            else decode_span_sync(l, w, limit, dcacc, E.sx, fetch, im.lut.data());
            SInfo r = {pack_state(l.p - limit, l.z, l.u), l.nb | (crossed << 31), pack_dc01(dcacc), pack_dc2(dcacc)};
            bool synced = r.x == E.sinfo[g].x;
            if (first && !synced) E.inter_changed++;
            first = false;
            E.sinfo[g] = r;
            ++g;
            if (synced || g >= gend) break;
        }
        E.warm[b + 1] = x0;
    }
}

// k_group_totals: does every sequence's set of records continue the state the sequence before it ends in?
void check_boundaries(Emul& E) {
    E.pending = 0;
    for (uint32_t b = 0; (uint64_t)(b + 1) * E.seq_len < E.im.nsub; ++b)
        if (E.warm[b + 1] != E.sinfo[(b + 1) * E.seq_len - 1].x) E.pending = 1;
}

void scan_and_write(Emul& E, int16_t* coef) {
    const Image& im = E.im;
    const uint32_t nsub = im.nsub, logL = E.logL, L = 1u << logL, wps = L >> 5;
    const uint32_t total = im.in.total_units;
    // poison: every coefficient has to be cleared by the group whose range holds it
    for (size_t k = 0; k < (size_t)total * 64; ++k) coef[k] = 0x5A5A;
    std::vector<uint8_t> cleared((size_t)total * 64, 0);
    const uint32_t* words = (const uint32_t*)im.stream.data();
    uint32_t unit0 = 0;
    int32_t pred[3] = {0, 0, 0};
    std::vector<uint32_t> strm;
    E.flags = 0;
    for (uint32_t i0 = 0; i0 < nsub; i0 += kWG) {
        const uint32_t nloc = std::min<uint32_t>(kWG, nsub - i0);
        const uint32_t first_word = i0 * wps, nwords = nloc * wps + 4;
        strm.assign(nwords, 0xDEADBEEF);
        for (uint32_t r = 0; r < nwords; ++r) strm[r] = bswap(words[first_word + r]);
        auto fetch = [&](uint32_t c) {
            if (c >= nwords) abort();
            return strm[c];
        };
        auto store = [&](uint32_t k, uint32_t at, int16_t v) {
            if (k >= total || at > 63) abort();
            coef[(size_t)k * 64 + at] = v;
        };
        const bool restart = im.in.restart_interval != 0;
        const uint32_t bm_k0 = first_word >> 3, bm_n = ((first_word + nwords + 7) >> 3) - bm_k0 + 1;
        auto bword = [&](uint32_t k) {
            if (k < bm_k0 || k - bm_k0 >= bm_n) abort();
            return im.bmap[k];
        };
        {
            uint32_t grp_units = 0;
            for (uint32_t t = 0; t < nloc; ++t) grp_units += rec_units(E.sinfo[i0 + t].y);
            const uint64_t end_all = (uint64_t)total * 64;
            const uint32_t x_in = i0 ? E.sinfo[i0 - 1].x : 0u, x_out = E.sinfo[i0 + nloc - 1].x;
            uint64_t a = (uint64_t)unit0 * 64 + state_z(x_in);
            uint64_t b = i0 + nloc >= nsub ? end_all : ((uint64_t)unit0 + grp_units) * 64 + state_z(x_out);
            if (i0 == 0) a = 0;
            if (b > end_all) b = end_all;
            for (uint64_t k = a; k < b; ++k) {
                if (cleared[k]) abort();  // ranges of different groups must not overlap
                cleared[k] = 1;
                coef[k] = 0;
            }
        }
        for (uint32_t t = 0; t < nloc; ++t) {
            const uint32_t i = i0 + t;
            const SInfo mine = E.sinfo[i];
            const uint32_t xprev = i ? E.sinfo[i - 1].x : 0u;
            Lane l;
            BitWin w;
            l.p = (i << logL) + state_prel(xprev); l.z = state_z(xprev); l.u = state_u(xprev); l.nb = 0;
            int32_t p0 = (int16_t)pred[0], p1 = (int16_t)pred[1], p2 = (int16_t)pred[2];
            uint32_t unit = unit0, flags = 0;
            if (unit < total && unit % im.in.units_per_mcu != l.u) flags |= kStUnit;
            const uint32_t limit = (i + 1) << logL;
            if (unit < total) {
                win_init(w, l.p, (l.p >> 5) - first_word, fetch);
                prime(l, w, E.sx, im.lut.data());
                if (restart) decode_span_write_rst(l, w, limit, unit, total, im.in.restart_interval * im.in.units_per_mcu, p0, p1, p2, E.sx, fetch, im.lut.data(), store, flags, bword);
                else decode_span_write(l, w, limit, unit, total, p0, p1, p2, E.sx, fetch, im.lut.data(), store, flags);
            }
            if (restart && i == 0) {
                const uint64_t mcus = (uint64_t)im.in.mcus_x * im.in.mcus_y;
                if (im.markers != (uint32_t)((mcus + im.in.restart_interval - 1) / im.in.restart_interval) - 1) flags |= kStInvalid;
            }
            if (unit < total) {
                if (l.p < limit || pack_state(l.p - limit, l.z, l.u) != mine.x) flags |= kStMismatch;
                if (i == nsub - 1) flags |= kStShort;
            }
            E.flags |= flags;
            // exclusive scan, lane by lane; the DC sums start afresh after a subsequence in which an interval began
            unit0 += rec_units(mine.y);
            if (rec_restarted(mine.y)) pred[0] = pred[1] = pred[2] = 0;
            pred[0] += sx16(mine.z); pred[1] += sx16(mine.z >> 16); pred[2] += sx16(mine.w);
        }
    }
}

void pixels(const Emul& E, const int16_t* coef_all, uint8_t* pix) {
    const jpgd_info& in = E.im.in;
    const uint8_t zz[64] = JPGD_ZIGZAG_LITERAL;
    const uint32_t upm = in.units_per_mcu, hs = in.hsamp[0], vs = in.vsamp[0], ncomp = in.ncomp;
    const uint32_t M = kPixBlocks / upm, runs = (in.mcus_x + M - 1) / M;
    const uint32_t mcu_w = 8 * hs, mcu_h = 8 * vs;
    std::vector<float> blk(kPixBlocks * 72);
    for (uint32_t mrow = 0; mrow < in.mcus_y; ++mrow)
        for (uint32_t run = 0; run < runs; ++run) {
            const uint32_t m0 = run * M, nm = std::min(M, in.mcus_x - m0), nblk = nm * upm;
            const int16_t* coef = coef_all + ((size_t)mrow * in.mcus_x + m0) * upm * 64;
            for (uint32_t k = 0; k < nblk; ++k) {
                uint32_t comp = (E.im.sched_comp >> ((k % upm) * 4)) & 15u;
                for (uint32_t zi = 0; zi < 64; ++zi)
                    blk[k * 72 + (zz[zi] >> 3) * 9 + (zz[zi] & 7)] = (float)coef[k * 64 + zi] * (float)in.qt[in.tq[comp]][zi];
            }
            for (uint32_t j = 0; j < nblk * 8; ++j) {
                float* b = &blk[(j >> 3) * 72 + (j & 7)];
                idct8(b[0], b[9], b[18], b[27], b[36], b[45], b[54], b[63]);
            }
            for (uint32_t j = 0; j < nblk * 8; ++j) {
                float* b = &blk[(j >> 3) * 72 + (j & 7) * 9];
                b[0] += kLevelShiftDc;
                idct8(b[0], b[1], b[2], b[3], b[4], b[5], b[6], b[7]);
            }
            for (uint32_t py = 0; py < mcu_h; ++py)
                for (uint32_t px = 0; px < nm * mcu_w; ++px) {
                    uint32_t gy = mrow * mcu_h + py, gx = m0 * mcu_w + px;
                    if (gy >= in.height || gx >= in.width) continue;
                    uint32_t m = px / mcu_w, xin = px % mcu_w;
                    float y = blk[(m * upm + (py >> 3) * hs + (xin >> 3)) * 72 + (py & 7) * 9 + (xin & 7)];
                    uint8_t* dst = pix + ((size_t)gy * in.width + gx) * ncomp;
                    if (ncomp == 1) { dst[0] = (uint8_t)pack_u8(y, 0u, 0u); continue; }
                    const float* cbb = &blk[(m * upm + hs * vs) * 72 + (py / vs) * 9];
                    const ChromaTerms c = chroma_terms(cbb[xin / hs], cbb[72 + xin / hs]);
                    dst[0] = (uint8_t)pack_u8(y + c.r, 0u, 0u);
                    dst[1] = (uint8_t)pack_u8(y + c.g, 0u, 0u);
                    dst[2] = (uint8_t)pack_u8(y + c.b, 0u, 0u);
                }
        }
}

}  // namespace

// Runs the whole pipeline on the host.  stats: [0] inter-sequence rounds used, [1] boundaries whose first
// comparison failed in the last round, [2] longest intra-sequence overflow (rounds), [3] final flags,
// [4] number of subsequences, [5] unstuffed bytes.  sinfo_out (may be NULL): 4 words per subsequence.
extern "C" int emul_decode(const uint8_t* file, size_t len, uint32_t L, uint32_t H, uint32_t max_rounds, int16_t* coef,
                           uint8_t* pix, uint32_t* sinfo_out, uint32_t sinfo_cap, uint8_t* stream_out,
                           uint32_t* stats) {
    Emul E;
    int rc = prepare(file, len, E.im);
    if (rc) return rc;
    E.logL = 0;
    while ((1u << E.logL) < L) ++E.logL;
    E.H = H;
    E.seq_len = kWG - H;
    for (uint32_t u = 0; u < E.im.in.units_per_mcu; ++u)
        E.rows[u] = make_unit_row(u, E.im.in.units_per_mcu, E.im.sched_dc, E.im.sched_ac, E.im.sched_comp);
    E.sx.rows = E.rows;
    E.sx.upm = E.im.in.units_per_mcu;
    E.sx.pair_of_unit = E.im.pair_of_unit;
    unstuff(file + E.im.in.scan_offset, (uint32_t)E.im.in.scan_bytes, E.logL, E.im);
    E.sinfo.assign(E.im.nsub, SInfo{0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu});
    const uint32_t nseq = (E.im.nsub + E.seq_len - 1) / E.seq_len;
    E.warm.assign(nseq + 1, 0xFFFFFFFFu);
    sync_intra(E);
    // as the host code of the library: everything once; if a boundary is still open, rounds that settle the
    // boundaries, then the write pass once more
    uint32_t rounds = 0;
    auto scan = [&]() {
        if (nseq > 1) { sync_inter(E); ++rounds; }
        check_boundaries(E);
    };
    scan();
    scan_and_write(E, coef);
    if (E.pending && nseq > 1 && rounds < max_rounds) {
        while (E.pending && rounds < max_rounds) scan();
        const bool open = E.pending != 0;
        scan_and_write(E, coef);
        if (open) E.flags |= kStMismatch;
    } else if (E.pending && nseq > 1) {
        E.flags |= kStMismatch;
    }
    if (stats) {
        stats[0] = rounds; stats[1] = E.inter_changed; stats[2] = E.rounds_max; stats[3] = E.flags;
        stats[4] = E.im.nsub; stats[5] = E.im.nbytes;
    }
    if (sinfo_out && sinfo_cap >= E.im.nsub) memcpy(sinfo_out, E.sinfo.data(), (size_t)E.im.nsub * 16);
    if (stream_out) memcpy(stream_out, E.im.stream.data(), E.im.nbytes);
    if (E.flags) return JPGD_E_CORRUPT;
    if (pix) pixels(E, coef, pix);
    return JPGD_OK;
}

// chains left at which the intra-sequence walk-through switches to the wavefront-per-chain decoder
extern "C" void emul_set_coop_max(uint32_t n) { g_coop_max = n; }
extern "C" void emul_set_sync_waves(uint32_t n) { g_sync_waves = n; }

// the literal zig-zag table of jpgd_idct.h, for comparison with a generated one
extern "C" void emul_zigzag(uint8_t out[64]) {
    const uint8_t zz[64] = JPGD_ZIGZAG_LITERAL;
    memcpy(out, zz, 64);
}

// one table built by jpgd_lut.h
extern "C" int emul_build_lut(const uint8_t* bits, const uint8_t* vals, int is_dc, uint16_t* out) {
    return build_lut(bits, vals, is_dc != 0, out) ? 0 : JPGD_E_TABLE;
}

// pair bytes of an AC table built by jpgd_lut.h (lut: the table's kLutEntries entries)
extern "C" void emul_build_pairs(const uint16_t* lut, uint8_t* pairs) { build_pairs(lut, pairs); }

// The synchronisation pass with two symbols per step against the one with single symbols, from decoder states that
// need not lie on the true chain: `nstart` starts at pseudo-random subsequences in pseudo-random states, each
// followed over `span` subsequences by both decoders (the lanes keep their window from one subsequence to the
// next, as in the kernel's overflow rounds).  Returns the number of subsequences after which the two disagreed in
// position, unit, zig-zag index, completed units or DC sums; stats[0] = steps of the single decoder,
// stats[1] = steps of the pair decoder over the same stretches.
extern "C" int emul_pairs_vs_single(const uint8_t* file, size_t len, uint32_t L, uint32_t nstart, uint32_t span,
                                    uint32_t seed, uint32_t* stats) {
    Emul E;
    int rc = prepare(file, len, E.im);
    if (rc) return -1;
    Image& im = E.im;
    if (im.in.restart_interval) return -1;
    E.logL = 0;
    while ((1u << E.logL) < L) ++E.logL;
    for (uint32_t u = 0; u < im.in.units_per_mcu; ++u)
        E.rows[u] = make_unit_row(u, im.in.units_per_mcu, im.sched_dc, im.sched_ac, im.sched_comp);
    E.sx.rows = E.rows;
    E.sx.upm = im.in.units_per_mcu;
    E.sx.pair_of_unit = im.pair_of_unit;
    unstuff(file + im.in.scan_offset, (uint32_t)im.in.scan_bytes, E.logL, im);
    const uint32_t* words = (const uint32_t*)im.stream.data();
    uint32_t steps[2] = {0u, 0u};
    int which = 0;
    auto fetch = [&](uint32_t w) { ++steps[which]; return bswap(words[w]); };  // one fetch per step (plus three per window)
    uint64_t rng = 0x9E3779B97F4A7C15ull ^ seed;
    auto next = [&]() { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return (uint32_t)(rng >> 16); };
    int bad = 0;
    if (im.nsub < 2) return 0;
    for (uint32_t k = 0; k < nstart; ++k) {
        const uint32_t i0 = next() % (im.nsub - 1u);
        const uint32_t prel = next() % 32u, z = next() % 64u, u = next() % im.in.units_per_mcu;
        Lane a, b;
        BitWin wa, wb;
        a.p = (i0 << E.logL) + prel; a.z = z; a.u = u; a.nb = 0;
        b = a;
        which = 0; win_init(wa, a.p, a.p >> 5, fetch); prime(a, wa, E.sx, im.lut.data());
        which = 1; win_init(wb, b.p, b.p >> 5, fetch); prime(b, wb, E.sx, im.lut.data());
        for (uint32_t i = i0; i < std::min(im.nsub, i0 + span); ++i) {
            const uint32_t limit = (i + 1u) << E.logL;
            int64_t da = 0, db = 0;
            a.nb = b.nb = 0;
            which = 0; decode_span_sync(a, wa, limit, da, E.sx, fetch, im.lut.data());
            which = 1; decode_span_sync_pairs(b, wb, limit, db, E.sx, fetch, im.lut.data(), im.pairs.data());
            if (a.p != b.p || a.u != b.u || a.z != b.z || a.nb != b.nb || da != db) { ++bad; break; }
        }
    }
    stats[0] = steps[0];
    stats[1] = steps[1];
    return bad;
}
