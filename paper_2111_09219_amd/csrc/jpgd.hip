// Host side of the decoder: workspace layout, per-call descriptors, kernel launches, the verdict.
// C ABI declared in include/jpgd.h.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <chrono>
#include <mutex>
#include <thread>
#include <vector>

#include "../../include/jpgd.h"
#include "jpgd_common.h"
#include "jpgd_kernels.h"
#include "jpgd_lut.h"

using namespace jpgd;

namespace {

constexpr uint32_t kMagic = 0x4A504744u;  // "JPGD"

// first bytes of the workspace: lets jpgd_read_sync_info find its way without the caller's help
struct WsHeader {
    uint32_t magic, nimg, logL, overlap;
    uint64_t off_status, off_state, off_img, off_lut, off_qt;       // uploaded region
    uint64_t off_tiles, off_stream, off_sinfo, off_gtot, off_gpref, off_bmap, off_warm, off_seqrec; // device-written regions
    uint64_t upload_bytes, total_bytes;
};

struct Plan {
    WsHeader h;
    std::vector<ImgDesc> img;
    std::vector<uint32_t> lut_of_img;  // index of the table set of image i
    uint32_t nsets = 0, lut_slots = 0, pair_slots = 0;
    uint32_t tiles = 0, seqs = 0, grps = 0, bnds = 0, pixwgs = 0, nsub_total = 0;
    uint32_t bmap_words = 0;  // interval-start bitmaps of the images that have restart intervals
    uint32_t L = 0;
    bool split = false;  // intra-sequence synchronisation as two kernels
};

size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

uint32_t ilog2(uint32_t v) {
    uint32_t l = 0;
    while ((1u << l) < v) ++l;
    return l;
}

bool same_tables(const jpgd_info& a, const jpgd_info& b) {
    if (a.ncomp != b.ncomp) return false;
    for (uint32_t c = 0; c < a.ncomp; ++c) {
        if (a.td[c] != b.td[c] || a.ta[c] != b.ta[c]) return false;
        if (memcmp(a.dht_bits[0][a.td[c]], b.dht_bits[0][b.td[c]], 16) ||
            memcmp(a.dht_vals[0][a.td[c]], b.dht_vals[0][b.td[c]], 256) ||
            memcmp(a.dht_bits[1][a.ta[c]], b.dht_bits[1][b.ta[c]], 16) ||
            memcmp(a.dht_vals[1][a.ta[c]], b.dht_vals[1][b.ta[c]], 256))
            return false;
    }
    return true;
}

// Subsequence size when the caller leaves it open.  The paper picks 1024 bits for high-quality material and
// 128 for short streams (Section 5, Tables II and III).  Two rules, the larger result counts:
//  * size: as large as possible (fewer overflow rounds, fewer records) while the call still has about 128k
//    subsequences to spread over the chip's 1024 SIMDs (measured on 4096x4096 grey and 4:4:4 streams of 2 to
//    24 MB and on batches of 1920x1088 images);
//  * content: a decoder needs a certain number of data units, not of bits, to fall into step - about 30 in a
//    4:4:4 or grey scan, about 140 in a 4:2:0 scan, where it also has to find its place among the six units of
//    the MCU - and a sequence of 240 subsequences must be several times that long, or most of its chains run
//    to its end without synchronising and the workgroup is no faster than one sequential decoder.  Measured
//    optimum: 2 (4:4:4, grey), 4 (4:2:2), 10 (4:2:0) times the scan's average bits per data unit, and never
//    below 256 bits for a subsampled scan.
// The size rule stops at four times what the content asks for: with sparse data units a lane of a large
// subsequence covers many units, the write pass's stores then come long after the clear of their lines, and
// large batches of sparse frames lose more in the write pass than they gain in the synchronisation (200 frames of
// 1920x1088 4:4:4, 148 MB at 60 bits per unit: 3.81 ms at 1024 bits, 3.58 at 512; 62 MB at 22 bits per unit:
// 3.13 ms at 1024 bits, 2.65 at 128).
uint32_t choose_subseq_bits(const jpgd_info* infos, int n) {
    uint64_t bits = 0;
    double want = 0.0;
    for (int i = 0; i < n; ++i) {
        const double b = (double)infos[i].scan_bytes * 8.0;
        const double per_unit = b / (double)(infos[i].total_units ? infos[i].total_units : 1u);
        const bool subsampled = infos[i].units_per_mcu >= 4u;
        const double factor = infos[i].units_per_mcu >= 6u ? 10.0 : subsampled ? 4.0 : 2.0;
        double w = factor * per_unit;
        if (subsampled && w < 256.0) w = 256.0;
        bits += infos[i].scan_bytes * 8u;
        want += b * w;
    }
    want /= (double)(bits ? bits : 1u);  // average over the call's bits
    uint32_t by_size = 128u, by_content = 128u;
    uint32_t cap = 128u;
    while (by_size < 1024u && bits / (2u * by_size) >= 131072u) by_size *= 2u;
    while (by_content < 1024u && want > 1.41 * (double)by_content) by_content *= 2u;
    while (cap < 1024u && 4.0 * want > 1.41 * (double)cap) cap *= 2u;
    if (by_size > cap) by_size = cap;
    return by_size > by_content ? by_size : by_content;
}

// Validates arguments that do not need the GPU and lays the workspace out.
int make_plan(const jpgd_info* infos, int n, const jpgd_config* cfg, Plan& pl) {
    if (!infos || n < 1) return JPGD_E_ARG;
    pl = Plan();  // (a slot's plan is used again by the slot's next call)
    const bool scaled = cfg && ((cfg->flags >> 2) & 3u) != 0u;  // reduced-size pixels: larger runs per workgroup
    uint32_t L = cfg && cfg->subseq_bits ? cfg->subseq_bits : choose_subseq_bits(infos, n);
    if (L < 128u || L > 2048u || (L & (L - 1u))) return JPGD_E_ARG;
    // default overlap: enough warm-up lanes that the chain entering a sequence is almost always synchronised,
    // which leaves the inter-sequence kernel one subsequence per boundary
    uint32_t H = (!cfg || cfg->overlap == 0xFFFFFFFFu) ? (L <= 256u ? 16u : 32u) : cfg->overlap;
    if (H > (uint32_t)kMaxOverlap) return JPGD_E_ARG;
    const uint32_t seq_len = kWG - H;
    pl.L = L;
    pl.img.assign(n, ImgDesc());
    pl.lut_of_img.assign(n, 0);
    size_t stream_bytes = 0;
    for (int i = 0; i < n; ++i) {
        const jpgd_info& in = infos[i];
        ImgDesc& d = pl.img[i];
        if (in.ncomp != 1 && in.ncomp != 3) return JPGD_E_ARG;
        if (in.units_per_mcu < 1 || in.units_per_mcu > 6 || kPixBlocks % in.units_per_mcu) return JPGD_E_ARG;
        if (in.scan_bytes < 1 || in.scan_bytes >= (1ull << 28)) return JPGD_E_ARG;
        if (in.total_units < 1 || in.total_units > 0x3FFFFFFu) return JPGD_E_ARG;
        d.scan_bytes = (uint32_t)in.scan_bytes;
        d.tile0 = pl.tiles;
        d.ntiles = (d.scan_bytes + kUnstuffTile - 1) / kUnstuffTile;
        pl.tiles += d.ntiles;
        d.restart = in.restart_interval;
        d.nint = 1;
        d.bmap_off = 0;
        if (d.restart) {
            const uint64_t mcus = (uint64_t)in.mcus_x * in.mcus_y;
            d.nint = (uint32_t)((mcus + d.restart - 1) / d.restart);
            d.bmap_off = pl.bmap_words;
            pl.bmap_words += d.ntiles * 128u + 128u;
        }
        d.stream_off = stream_bytes;
        stream_bytes += up256((size_t)d.scan_bytes + L / 8 + 64 + 16);
        d.nsub_max = (uint32_t)(((uint64_t)d.scan_bytes * 8 + L - 1) / L);
        d.sub0 = pl.nsub_total;
        pl.nsub_total += (d.nsub_max + 3u) & ~3u;
        d.seq0 = pl.seqs;
        d.nseq_max = (d.nsub_max + seq_len - 1) / seq_len;
        pl.seqs += d.nseq_max;
        d.grp0 = pl.grps;
        d.ngrp_max = (d.nsub_max + kWG - 1) / kWG;
        pl.grps += d.ngrp_max;
        d.bnd0 = pl.bnds;
        d.nbnd_wg = d.nseq_max > 1 ? (d.nseq_max - 1 + 63) / 64 : 0;
        pl.bnds += d.nbnd_wg;
        d.total_units = in.total_units;
        d.upm = in.units_per_mcu;
        d.width = in.width; d.height = in.height; d.ncomp = in.ncomp;
        d.hs = in.hsamp[0]; d.vs = in.vsamp[0];
        d.mcus_x = in.mcus_x; d.mcus_y = in.mcus_y;
        if (d.upm != (in.ncomp == 1 ? 1u : d.hs * d.vs + 2u)) return JPGD_E_ARG;
        if ((uint64_t)d.mcus_x * d.mcus_y * d.upm != d.total_units) return JPGD_E_ARG;
        const uint32_t M = (uint32_t)(scaled ? kPixBlocksScaled : kPixBlocks) / d.upm;
        d.pix_runs = (d.mcus_x + M - 1) / M;
        d.pix_wg0 = pl.pixwgs;
        if ((uint64_t)pl.pixwgs + (uint64_t)d.pix_runs * d.mcus_y > 0x7FFFFFFFull) return JPGD_E_ARG;  // grid size
        pl.pixwgs += d.pix_runs * d.mcus_y;
        // table slots: distinct DC tables first, then distinct AC tables, in order of first use
        uint32_t dc_ids[3], ac_ids[3], ndc = 0, nac = 0, comp_dc[3], comp_ac[3];
        for (uint32_t c = 0; c < in.ncomp; ++c) {
            if (in.td[c] > 3 || in.ta[c] > 3 || !in.dht_present[0][in.td[c]] || !in.dht_present[1][in.ta[c]] ||
                in.tq[c] > 3 || !in.qt_present[in.tq[c]])
                return JPGD_E_TABLE;
            uint32_t k;
            for (k = 0; k < ndc && dc_ids[k] != in.td[c]; ++k) {}
            if (k == ndc) dc_ids[ndc++] = in.td[c];
            comp_dc[c] = k;
            for (k = 0; k < nac && ac_ids[k] != in.ta[c]; ++k) {}
            if (k == nac) ac_ids[nac++] = in.ta[c];
            comp_ac[c] = k;
        }
        d.nslots = ndc + nac;
        d.ndc = ndc;
        if (nac > pl.pair_slots) pl.pair_slots = nac;
        d.sched_dc = d.sched_ac = d.sched_comp = 0;
        uint32_t u = 0;
        for (uint32_t c = 0; c < in.ncomp; ++c) {
            uint32_t nu = c == 0 ? d.hs * d.vs : 1u;
            if (in.ncomp == 1) nu = 1;
            for (uint32_t k = 0; k < nu; ++k, ++u) {
                d.sched_dc |= comp_dc[c] << (4 * u);
                d.sched_ac |= (ndc + comp_ac[c]) << (4 * u);
                d.sched_comp |= c << (4 * u);
            }
        }
        if (u != d.upm) return JPGD_E_ARG;
        if (i > 0 && same_tables(infos[i - 1], in)) {
            pl.lut_of_img[i] = pl.lut_of_img[i - 1];
        } else {
            pl.lut_of_img[i] = pl.nsets++;
        }
        if (d.nslots > pl.lut_slots) pl.lut_slots = d.nslots;
    }
    for (int i = 0; i < n; ++i) {
        pl.img[i].lut_off = pl.lut_of_img[i] * (uint32_t)kLutSetEntries;
        pl.img[i].qt_off = (uint32_t)i * 192u;
    }
    if (pl.nsub_total > 0x7FFFFFF0u || pl.tiles > 0x7FFFFFF0u) return JPGD_E_ARG;
    // Intra-sequence synchronisation in two kernels: when the call has many more sequences than the chip holds at a
    // time (three per CU with 1024-bit subsequences staged in LDS) and the staged stream is what limits that number.
    // Measured on the 15360x8640 image (2320 sequences): 2.80 -> 2.65 ms per call; on calls the chip holds at once
    // the second kernel only adds its launch.
    {
        const uint32_t mode = cfg ? cfg->sync_split : 0u;
        if (mode > 2u) return JPGD_E_ARG;
        // (not with restart intervals: their second kernel, with one chain per wavefront at most and single-symbol
        // steps, takes longer than it saves -- 15360x8640 with one interval per MCU row 2.13 against 2.10 ms)
        const bool can = pl.bmap_words == 0u && pl.lut_slots <= 4u;
        pl.split = can && (mode == 2u || (mode == 0u && L >= 512u && pl.seqs >= (uint32_t)kSplitMinSeqs));
    }

    WsHeader& h = pl.h;
    memset(&h, 0, sizeof h);
    h.magic = kMagic; h.nimg = (uint32_t)n; h.logL = ilog2(L); h.overlap = H;
    size_t off = up256(sizeof(WsHeader));
    h.off_status = off; off = up256(off + sizeof(Status));
    h.off_state = off;  off = up256(off + sizeof(ImgState) * (size_t)n);
    h.off_img = off;    off = up256(off + sizeof(ImgDesc) * (size_t)n);
    h.off_lut = off;    off = up256(off + (size_t)pl.nsets * kLutSetEntries * 2);
    h.off_qt = off;     off = up256(off + (size_t)n * 192 * 2);
    h.upload_bytes = off;
    h.off_tiles = off;  off = up256(off + (size_t)pl.tiles * 4);
    h.off_stream = off; off = up256(off + stream_bytes);
    h.off_sinfo = off;  off = up256(off + (size_t)pl.nsub_total * sizeof(SInfo));
    h.off_gtot = off;   off = up256(off + (size_t)pl.grps * 16);
    h.off_gpref = off;  off = up256(off + (size_t)pl.grps * 16);
    h.off_bmap = off;   off = up256(off + (size_t)pl.bmap_words * 4);
    h.off_warm = off;   off = up256(off + (size_t)pl.seqs * 4);
    h.off_seqrec = off; off = up256(off + (pl.split ? (size_t)pl.seqs * kHandWords * 4u : 0u));
    h.total_bytes = off;
    return JPGD_OK;
}

// ---- one decode call between its enqueue and its wait ---------------------------------------------------
// Per call: a pinned buffer for the parameter block and a pinned, coherent 64-byte block for the verdict.  Both are
// reached from the GPU directly: a small kernel (or a few extra workgroups of the first kernel) copies the parameters
// into the workspace and the first lane of the pixel kernel reports the verdict, so that nothing but kernels sits in
// the stream (a copy engine between two kernels, or an event, costs several microseconds of an otherwise idle GPU
// each).  Calls in flight each hold a slot of their own, so that a host thread can enqueue the next batch while the
// GPU still works on this one (the paper's end-to-end setting, Section 5: transfers and decoding of consecutive
// batches overlap), and two threads never wait for each other.
constexpr int kMaxDevices = 16;
constexpr size_t kStaticWsBytes = (size_t)JPGD_STATIC_WORKSPACE_BYTES;
constexpr size_t kStaticStageBytes = 64 * 1024;  // parameter block of one image: 24 KB (the tables take 21 KB of it whatever their number)

struct Timed { int kernel; size_t ev; };

}  // namespace

struct jpgd_call {
    // owned for the life of the process
    int device = -1;
    uint8_t* buf = nullptr;        // pinned
    uint8_t* buf_dev = nullptr;    // the same bytes as the device addresses them
    size_t cap = 0;
    uint32_t* verdict = nullptr;   // pinned, 16 words: [0] flags, [1] inter_changed, [2] pending, [15] ticket of the report
    uint32_t* verdict_dev = nullptr;
    uint32_t ticket = 0;
    std::vector<hipEvent_t> timers;  // pairs of events for timing_mask
    bool busy = false;
    bool fixed = false;            // the slot of the entry point that allocates nothing: never grown, never shared
    bool launched = false;         // something of the current call is in the stream
    // the call in flight
    Plan pl;
    Params P;
    hipStream_t stream = nullptr;
    uint8_t* ws = nullptr;
    bool want_pixels = false, staged = false, big_groups = false;
    int variant = 0;
    size_t lds_sync = 0, lds_write = 0, lds_inter = 0;
    uint32_t tmask = 0, max_rounds = 0, rounds = 0, redo = 0;
    std::vector<Timed> timed;
    uint32_t launches[JPGD_N_KERNELS] = {0};
};

namespace {

using Call = jpgd_call;

std::mutex g_mu;                 // guards the slot list, the table cache and the per-device bookkeeping; never held
                                 // while the GPU is waited for
std::vector<Call*> g_calls;
constexpr size_t kMaxCalls = 64;

int hip_failed(const char* what, hipError_t e) {
    fprintf(stderr, "jpgd: %s failed: %s\n", what, hipGetErrorString(e));
    return JPGD_E_HIP;
}
#define HIP_OK(expr)                                                \
    do {                                                            \
        hipError_t e_ = (expr);                                     \
        if (e_ != hipSuccess) return hip_failed(#expr, e_);         \
    } while (0)

int call_reserve(Call& c, size_t bytes) {
    if (c.cap < bytes) {
        if (c.fixed) return JPGD_E_WORKSPACE;
        if (c.buf) (void)hipHostFree(c.buf);
        c.buf = c.buf_dev = nullptr;
        c.cap = 0;
        const size_t want = bytes + (bytes >> 2) + 4096;
        HIP_OK(hipHostMalloc((void**)&c.buf, want, hipHostMallocMapped));
        HIP_OK(hipHostGetDevicePointer((void**)&c.buf_dev, c.buf, 0));
        c.cap = want;
    }
    if (!c.verdict) {
        if (c.fixed) return JPGD_E_WORKSPACE;
        HIP_OK(hipHostMalloc((void**)&c.verdict, 64, hipHostMallocMapped | hipHostMallocCoherent));
        HIP_OK(hipHostGetDevicePointer((void**)&c.verdict_dev, c.verdict, 0));
        memset(c.verdict, 0, 64);
    }
    return JPGD_OK;
}

// a free slot of the current device (a new one if all are in flight)
int call_acquire(Call** out) {
    int dev = 0;
    HIP_OK(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mu);
    for (Call* c : g_calls)
        if (!c->busy && !c->fixed && c->device == dev) {
            c->busy = true;
            *out = c;
            return JPGD_OK;
        }
    if (g_calls.size() >= kMaxCalls) return JPGD_E_BUSY;
    Call* c = new Call();
    c->device = dev;
    c->busy = true;
    g_calls.push_back(c);
    *out = c;
    return JPGD_OK;
}

void call_release(Call* c) {
    std::lock_guard<std::mutex> lock(g_mu);
    c->busy = false;
}

__global__ __launch_bounds__(kWG) void k_upload(const uint4* __restrict__ src, uint4* __restrict__ dst, uint32_t n16) {
    for (uint32_t k = blockIdx.x * kWG + threadIdx.x; k < n16; k += gridDim.x * kWG) dst[k] = src[k];
}

// one lane: status words to the host, then the ticket the host is waiting for
__global__ void k_verdict(const Status* st, volatile uint32_t* host, uint32_t ticket) {
    if (threadIdx.x == 0) {
        host[0] = st->flags;
        host[1] = st->inter_changed;
        host[2] = st->pending;
        __threadfence_system();
        host[15] = ticket;
    }
}

// The status words go back to zero before a further round.  A kernel, not a memset: callers may capture the
// stream, and the rest of the path is kernels only.
__global__ void k_clear_status(Status* st) {
    if (threadIdx.x == 0) {
        st->flags = 0u;
        st->inter_changed = 0u;
        st->pending = 0u;
        st->pad = 0u;
    }
}

// Lookup tables built recently, keyed by the DHT lists they came from: most files share a handful of
// tables (the typical ones of the standard above all), and building one costs a few microseconds of a
// call that may take a hundred.  Guarded by g_lut_mu.
struct LutCacheEntry {
    bool is_dc;
    uint8_t bits[16];
    uint8_t vals[256];
    uint32_t nvals;
    uint64_t stamp;
    uint16_t lut[kLutEntries];
    uint8_t pairs[kPairBytes];  // AC tables
};
std::mutex g_lut_mu;
std::vector<LutCacheEntry> g_lut_cache;
uint64_t g_lut_clock = 0;
constexpr size_t kLutCacheMax = 32;

// pairs: where the pair bytes of an AC table go (null for a DC table)
bool cached_lut(const uint8_t bits[16], const uint8_t* vals, bool is_dc, uint16_t* out, uint8_t* pairs) {
    uint32_t nvals = 0;
    for (int k = 0; k < 16; ++k) nvals += bits[k];
    if (nvals > 256u) return false;
    std::lock_guard<std::mutex> lock(g_lut_mu);
    for (LutCacheEntry& e : g_lut_cache)
        if (e.is_dc == is_dc && e.nvals == nvals && !memcmp(e.bits, bits, 16) && !memcmp(e.vals, vals, nvals)) {
            e.stamp = ++g_lut_clock;
            memcpy(out, e.lut, sizeof e.lut);
            if (pairs) memcpy(pairs, e.pairs, sizeof e.pairs);
            return true;
        }
    if (!build_lut(bits, vals, is_dc, out)) return false;
    if (pairs) build_pairs(out, pairs);
    LutCacheEntry* victim;
    if (g_lut_cache.size() < kLutCacheMax) {
        g_lut_cache.emplace_back();
        victim = &g_lut_cache.back();
    } else {
        victim = &g_lut_cache[0];
        for (LutCacheEntry& e : g_lut_cache)
            if (e.stamp < victim->stamp) victim = &e;  // least recently used
    }
    victim->is_dc = is_dc;
    memcpy(victim->bits, bits, 16);
    memcpy(victim->vals, vals, nvals);
    victim->nvals = nvals;
    victim->stamp = ++g_lut_clock;
    memcpy(victim->lut, out, sizeof victim->lut);
    if (pairs) memcpy(victim->pairs, pairs, sizeof victim->pairs);
    return true;
}

// Waits until the verdict has been reported under `ticket`.  A short decode is answered within microseconds, so the
// wait starts as a spin on the pinned word; after 50 microseconds the thread yields between looks and after 2 ms it
// sleeps, so that a long decode does not cost a busy core.  The stream is asked now and then, so that a failed
// launch or a lost report ends the wait with an error instead of hanging.
int wait_verdict(Call& c) {
    volatile uint32_t* v = c.verdict;
    const auto t0 = std::chrono::steady_clock::now();
    int64_t waited_us = 0;
    for (uint32_t looks = 1;; ++looks) {
        if (v[15] == c.ticket) break;
        if (waited_us < 50) {
            if ((looks & 63u) == 0u)
                waited_us = std::chrono::duration_cast<std::chrono::microseconds>(std::chrono::steady_clock::now() - t0).count();
            continue;
        }
        waited_us = std::chrono::duration_cast<std::chrono::microseconds>(std::chrono::steady_clock::now() - t0).count();
        if (waited_us < 2000) std::this_thread::yield();
        else std::this_thread::sleep_for(std::chrono::microseconds(50));
        if ((looks & 0xFFu) == 0u) {
            hipError_t q = hipStreamQuery(c.stream);
            if (q == hipSuccess) {
                if (v[15] == c.ticket) break;
                fprintf(stderr, "jpgd: the stream is idle but the verdict has not arrived\n");
                return JPGD_E_HIP;
            }
            if (q != hipErrorNotReady) return hip_failed("hipStreamQuery", q);
        }
    }
    __atomic_thread_fence(__ATOMIC_ACQUIRE);
    return JPGD_OK;
}

// subsequences of up to this many bits are staged in LDS by the sync and write kernels
// (JPGD_STAGED_MAX_BITS overrides it for tuning runs)
uint32_t staged_max_bits() {
    static const uint32_t v = [] {
        const char* e = getenv("JPGD_STAGED_MAX_BITS");
        return e ? (uint32_t)atoi(e) : 2048u;
    }();
    return v;
}
#define kStagedMaxL staged_max_bits()

// with restart intervals the kernels also keep the interval-start bitmap of the staged bytes: one bit per byte
size_t lds_bitmap_bytes(uint32_t L, bool restart) {
    return restart && L <= (uint32_t)kBitmapLdsMaxL ? ((size_t)(kWG * (L / 32) + 4 + 7) / 8 + 2) * 4 : 0;
}
size_t lds_sync_bytes(uint32_t L, uint32_t lut_slots, uint32_t pair_slots, bool restart) {
    uint32_t nwords = L <= kStagedMaxL ? kWG * (L / 32) + 4 : 4;
    return (size_t)lut_slots * kLutEntries * 2 + (size_t)pair_slots * kPairBytes + 6 * kWG * 4 + (size_t)nwords * 4 +
           lds_bitmap_bytes(L, restart);
}
// the second of the two synchronisation kernels keeps the tables and the records, not the stream
size_t lds_tail_bytes(uint32_t lut_slots, uint32_t pair_slots) {
    return (size_t)lut_slots * kLutEntries * 2 + (size_t)pair_slots * kPairBytes + 4 * kWG * 4 + 2 * kHandMax * 4 + 16;
}
size_t lds_write_bytes(uint32_t L, uint32_t lut_slots, bool restart) {
    uint32_t nwords = L <= kStagedMaxL ? kWG * (L / 32) + 4 : 4;
    return (size_t)lut_slots * kLutEntries * 2 + (size_t)nwords * 4 + lds_bitmap_bytes(L, restart);
}

// dynamic LDS beyond the default limit has to be requested per kernel and device; remember what was granted
size_t g_lds_granted[kMaxDevices][9];
int grant_lds(int dev, int which, const void* kernel, size_t bytes) {
    if (bytes <= 48 * 1024) return JPGD_OK;
    std::lock_guard<std::mutex> lock(g_mu);
    if (dev < 0 || dev >= kMaxDevices) return JPGD_E_ARG;
    if (bytes <= g_lds_granted[dev][which]) return JPGD_OK;
    HIP_OK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    g_lds_granted[dev][which] = bytes;
    return JPGD_OK;
}

// ---- launches ---------------------------------------------------------------------------------------

int t_begin(Call& c, int k) {
    c.launches[k]++;
    if (!(c.tmask & (1u << k))) return JPGD_OK;
    const size_t need = 2 * (c.timed.size() + 1);
    while (c.timers.size() < need) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return JPGD_E_HIP;
        c.timers.push_back(e);
    }
    c.timed.push_back({k, 2 * c.timed.size()});
    return hipEventRecord(c.timers[c.timed.back().ev], c.stream) == hipSuccess ? JPGD_OK : JPGD_E_HIP;
}
int t_end(Call& c, int k) {
    if (!(c.tmask & (1u << k))) return JPGD_OK;
    return hipEventRecord(c.timers[c.timed.back().ev + 1], c.stream) == hipSuccess ? JPGD_OK : JPGD_E_HIP;
}
#define LAUNCH(K, kernel, grid, block, lds)                                       \
    do {                                                                          \
        int rc_ = t_begin(c, K);                                                  \
        if (rc_ != JPGD_OK) return rc_;                                           \
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(block), lds, c.stream, c.P);  \
        if ((rc_ = t_end(c, K)) != JPGD_OK) return rc_;                           \
    } while (0)

// inter-sequence round, group totals, prefix of the totals
int launch_scan(Call& c) {
    if (c.pl.bnds) {
        LAUNCH(JPGD_K_SYNC_INTER, k_sync_inter, c.pl.bnds, 64, c.lds_inter);
        ++c.rounds;
    }
    LAUNCH(JPGD_K_SCAN_TOTALS, k_group_totals, c.pl.grps, kWG, 0);
    if (c.big_groups) LAUNCH(JPGD_K_SCAN_PREFIX, k_group_scan, c.pl.h.nimg, kWG, 0);
    return JPGD_OK;
}

int launch_write(Call& c) {
    if (c.staged) LAUNCH(JPGD_K_WRITE, k_write<true>, c.pl.grps, kWG, c.lds_write);
    else LAUNCH(JPGD_K_WRITE, k_write<false>, c.pl.grps, kWG, c.lds_write);
    return JPGD_OK;
}

// The pixel kernel is enqueued before the verdict is known: it only reads coefficients, and if the verdict is bad
// its output is either redone or reported as unspecified.  Its first lane passes the verdict on before anything
// else; the host waits for the verdict alone, and the pixels are complete in stream order, like the output of any
// kernel.  Without pixels a one-lane kernel reports.
int launch_report(Call& c, bool with_pixels) {
    const uint32_t ticket = ++c.ticket;
    if (with_pixels) {
        c.P.verdict = c.verdict_dev;
        c.P.ticket = ticket;
        if (c.P.scale_log2 == 0u) LAUNCH(JPGD_K_PIXELS, k_pixels, c.pl.pixwgs, kWG, 0);
        else if (c.P.scale_log2 == 1u) LAUNCH(JPGD_K_PIXELS, k_pixels_scaled<4>, c.pl.pixwgs, kWG, 0);
        else if (c.P.scale_log2 == 2u) LAUNCH(JPGD_K_PIXELS, k_pixels_scaled<2>, c.pl.pixwgs, kWG, 0);
        else LAUNCH(JPGD_K_PIXELS, k_pixels_scaled<1>, c.pl.pixwgs, kWG, 0);
    } else {
        hipLaunchKernelGGL(k_verdict, dim3(1), dim3(64), 0, c.stream, (const Status*)(c.ws + c.pl.h.off_status),
                           (volatile uint32_t*)c.verdict_dev, ticket);
    }
    HIP_OK(hipGetLastError());
    return JPGD_OK;
}

// Everything of a call up to and including its first report: validation, plan, parameter block, all kernels.
// Nothing here waits for the GPU.  ws_cap: bytes behind d_workspace.
int enqueue_call(Call& c, int n, const jpgd_info* infos, const uint8_t* d_scans, const uint64_t* scan_offsets,
                 int16_t* d_coef, const uint64_t* coef_offsets, uint8_t* d_pixels, const uint64_t* pixel_offsets,
                 void* d_workspace, size_t ws_cap, const jpgd_config* cfg, hipStream_t stream) {
    Plan& pl = c.pl;
    int rc = make_plan(infos, n, cfg, pl);
    if (rc) return rc;
    if (ws_cap < pl.h.total_bytes) return JPGD_E_WORKSPACE;
    const uint32_t flags_in = cfg ? cfg->flags : 0u;
    const uint32_t scale_log2 = (flags_in >> 2) & 3u;  // JPGD_F_SCALE_2, _4, _8 = 1, 2, 3 in bits 2..3
    c.want_pixels = d_pixels && !(flags_in & JPGD_F_NO_PIXELS);
    for (int i = 0; i < n; ++i) {
        if (scan_offsets[i] & 15u) return JPGD_E_ARG;
        if (coef_offsets[i] & 63u) return JPGD_E_ARG;
        pl.img[i].scan_off = scan_offsets[i];
        pl.img[i].coef_off = coef_offsets[i];
        pl.img[i].pix_off = c.want_pixels ? pixel_offsets[i] : 0;
    }
    c.stream = stream;
    c.ws = (uint8_t*)d_workspace;
    const bool any_restart = pl.bmap_words != 0u;
    c.lds_sync = lds_sync_bytes(pl.L, pl.lut_slots, pl.pair_slots, any_restart);
    c.lds_write = lds_write_bytes(pl.L, pl.lut_slots, any_restart);
    c.lds_inter = (size_t)pl.lut_slots * kLutEntries * 2;
    if (c.lds_sync > 150 * 1024) return JPGD_E_ARG;
    c.staged = pl.L <= kStagedMaxL;
    // the variants of the intra-sequence kernel: stream staged in LDS or not, call with or without restart intervals
    c.variant = (c.staged ? 0 : 1) + (any_restart ? 2 : 0);
    const void* const sync_kernels[4] = {(const void*)k_sync_intra<true, false>, (const void*)k_sync_intra<false, false>,
                                         (const void*)k_sync_intra<true, true>, (const void*)k_sync_intra<false, true>};
    if ((rc = grant_lds(c.device, c.variant, sync_kernels[c.variant], c.lds_sync)) ||
        (rc = grant_lds(c.device, c.staged ? 4 : 5, c.staged ? (const void*)k_write<true> : (const void*)k_write<false>, c.lds_write)) ||
        (rc = grant_lds(c.device, 8, (const void*)k_sync_inter, c.lds_inter)) ||
        (pl.split && c.staged && (rc = grant_lds(c.device, 6, (const void*)k_sync_head<true, false>, c.lds_sync))))
        return rc;
    rc = call_reserve(c, pl.h.upload_bytes + 16);
    if (rc) return rc;
    uint8_t* up = c.buf;
    memset(up, 0, pl.h.upload_bytes);
    memcpy(up, &pl.h, sizeof pl.h);
    memcpy(up + pl.h.off_img, pl.img.data(), sizeof(ImgDesc) * (size_t)n);
    uint16_t* luts = (uint16_t*)(up + pl.h.off_lut);
    uint16_t* qts = (uint16_t*)(up + pl.h.off_qt);
    for (int i = 0; i < n; ++i) {
        const jpgd_info& in = infos[i];
        const ImgDesc& d = pl.img[i];
        if (i == 0 || pl.lut_of_img[i] != pl.lut_of_img[i - 1]) {
            uint16_t* set = luts + d.lut_off;
            uint32_t built = 0u;  // slots of this set already filled
            for (uint32_t u = 0; u < d.upm; ++u) {
                uint32_t cc = (d.sched_comp >> (4 * u)) & 15u;
                uint32_t sd = (d.sched_dc >> (4 * u)) & 15u, sa = (d.sched_ac >> (4 * u)) & 15u;
                if (!(built & (1u << sd)) &&
                    !cached_lut(in.dht_bits[0][in.td[cc]], in.dht_vals[0][in.td[cc]], true, set + sd * kLutEntries, nullptr))
                    return JPGD_E_TABLE;
                built |= 1u << sd;
                if (!(built & (1u << sa)) &&
                    !cached_lut(in.dht_bits[1][in.ta[cc]], in.dht_vals[1][in.ta[cc]], false, set + sa * kLutEntries,
                                (uint8_t*)(set + kMaxSlots * kLutEntries) + (sa - d.ndc) * kPairBytes))
                    return JPGD_E_TABLE;
                built |= 1u << sa;
            }
        }
        for (uint32_t cc = 0; cc < in.ncomp; ++cc)
            for (int k = 0; k < 64; ++k) qts[d.qt_off + cc * 64 + k] = in.qt[in.tq[cc]][k];
    }
    uint8_t* ws = c.ws;
    // The parameter block goes from the pinned buffer into the workspace: for a batch by a kernel of its own (the
    // first kernel of the path already looks its image up in the block), for a single image by extra workgroups of
    // that first kernel, which then finds all it needs in its arguments.
    const uint32_t up_n16 = (uint32_t)((pl.h.upload_bytes + 15u) / 16u);
    uint32_t up_wgs = (up_n16 + kWG - 1u) / kWG;
    if (up_wgs > 256u) up_wgs = 256u;

    Params& P = c.P;
    P.img = (const ImgDesc*)(ws + pl.h.off_img);
    P.st = (ImgState*)(ws + pl.h.off_state);
    P.status = (Status*)(ws + pl.h.off_status);
    P.scans = d_scans;
    P.stream = ws + pl.h.off_stream;
    P.tile_cnt = (uint32_t*)(ws + pl.h.off_tiles);
    P.sinfo = (SInfo*)(ws + pl.h.off_sinfo);
    P.grp_tot = (int4*)(ws + pl.h.off_gtot);
    P.grp_pref = (int4*)(ws + pl.h.off_gpref);
    P.bmap = (uint32_t*)(ws + pl.h.off_bmap);
    P.warm_x = (uint32_t*)(ws + pl.h.off_warm);
    P.seq_rec = (uint32_t*)(ws + pl.h.off_seqrec);
    P.luts = (const uint16_t*)(ws + pl.h.off_lut);
    P.qts = (const uint16_t*)(ws + pl.h.off_qt);
    P.coef = d_coef;
    P.pixels = d_pixels;
    P.nimg = (uint32_t)n;
    P.logL = pl.h.logL;
    P.overlap = pl.h.overlap;
    P.seq_len = kWG - pl.h.overlap;
    P.lut_slots = pl.lut_slots;
    P.pair_slots = pl.pair_slots;
    P.planar = (flags_in & JPGD_F_PLANAR) ? 1u : 0u;
    P.scale_log2 = scale_log2;
    // Wavefronts per workgroup of the intra-sequence kernel: as many as the CU's 32 slots allow beside the other
    // workgroups it will hold (LDS, or the size of the grid, decides how many those are), at most 16; more than
    // 8 only pay when a round is long (measured: 16 instead of 8 gains 5 % at 1024 bits, nothing at 128).  Calls
    // with restart intervals stay at four: their kernel needs twice the registers.
    uint32_t sync_waves = (uint32_t)(kWG / 64);
    {
        const uint32_t slots = any_restart ? 20u : 32u;  // the kernel for restart intervals needs 92 registers: 5 per SIMD
        const uint32_t by_lds = (uint32_t)(160u * 1024u / c.lds_sync), by_grid = (pl.seqs + 255u) / 256u;
        const uint32_t per_cu = by_lds < by_grid ? (by_lds ? by_lds : 1u) : by_grid;
        const uint32_t most = pl.L >= 512u ? (uint32_t)kSyncWavesMax : 8u;
        while (sync_waves * 2u <= most && sync_waves * 2u * per_cu <= slots) sync_waves *= 2u;
    }
    P.sync_waves = sync_waves;
    P.coop_max = kCoopMax * sync_waves / (uint32_t)(kWG / 64);
    P.handoff = 0u;
    P.verdict = nullptr;
    P.ticket = 0u;
    P.up_src = (const uint4*)c.buf_dev;
    P.up_dst = (uint4*)ws;
    P.up_n16 = up_n16;
    P.up_wgs = n > 1 ? 0u : up_wgs;
    P.img0 = pl.img[0];

    c.tmask = cfg ? cfg->timing_mask : 0u;
    c.timed.clear();
    memset(c.launches, 0, sizeof c.launches);
    c.rounds = c.redo = 0u;
    c.max_rounds = cfg && cfg->max_rounds ? cfg->max_rounds : pl.seqs + 1;

    c.launched = true;
    if (n > 1)
        hipLaunchKernelGGL(k_upload, dim3(up_wgs), dim3(kWG), 0, stream, (const uint4*)c.buf_dev, (uint4*)ws, up_n16);
    LAUNCH(JPGD_K_UNSTUFF_COUNT, k_unstuff_count, pl.tiles + P.up_wgs, kWG, 0);
    P.up_wgs = 0u;
    bool big_tiles = false;  // the two image-level scans are only needed beyond 256 tiles / groups
    c.big_groups = false;
    for (int i = 0; i < n; ++i) {
        big_tiles = big_tiles || pl.img[i].ntiles > (uint32_t)kWG;
        c.big_groups = c.big_groups || pl.img[i].ngrp_max > (uint32_t)kWG;
    }
    if (big_tiles) LAUNCH(JPGD_K_UNSTUFF_SCAN, k_unstuff_scan, n, kWG, 0);
    LAUNCH(JPGD_K_UNSTUFF_SCATTER, k_unstuff_scatter, pl.tiles, kWG, 0);
    if (pl.split) {
        // first kernel: until at most kHandoff chains of a sequence are left; second kernel: the rest, four
        // wavefronts per sequence, the chains from kCoopMax down one per wavefront
        P.handoff = kHandoff;
        if (c.staged) LAUNCH(JPGD_K_SYNC_INTRA, (k_sync_head<true, false>), pl.seqs, kWG, c.lds_sync);
        else LAUNCH(JPGD_K_SYNC_INTRA, (k_sync_head<false, false>), pl.seqs, kWG, c.lds_sync);
        P.sync_waves = (uint32_t)(kWG / 64);
        P.coop_max = kCoopMax;
        LAUNCH(JPGD_K_SYNC_TAIL, (k_sync_tail<false>), pl.seqs, kWG, lds_tail_bytes(pl.lut_slots, pl.pair_slots));
    } else
    switch (c.variant) {
        case 0: LAUNCH(JPGD_K_SYNC_INTRA, (k_sync_intra<true, false>), pl.seqs, 64u * P.sync_waves, c.lds_sync); break;
        case 1: LAUNCH(JPGD_K_SYNC_INTRA, (k_sync_intra<false, false>), pl.seqs, 64u * P.sync_waves, c.lds_sync); break;
        case 2: LAUNCH(JPGD_K_SYNC_INTRA, (k_sync_intra<true, true>), pl.seqs, 64u * P.sync_waves, c.lds_sync); break;
        default: LAUNCH(JPGD_K_SYNC_INTRA, (k_sync_intra<false, true>), pl.seqs, 64u * P.sync_waves, c.lds_sync); break;
    }
    // Everything is launched in one go, write pass and pixels included: nearly every call is settled by one
    // inter-sequence round, and the host need not hear from the GPU in between.
    if ((rc = launch_scan(c)) || (rc = launch_write(c)) || (rc = launch_report(c, c.want_pixels))) return rc;
    return JPGD_OK;
}

// Waits for the verdict of a call and, if the boundaries between sequences are not settled yet, settles them first
// (rounds of the inter-sequence kernel and the totals kernel, which says whether a boundary is still open; paper: the
// host repeats the phase until all sequences are synchronised) and runs the write pass and the pixels once more.
int finish_call(Call& c, jpgd_report* report) {
    int rc = wait_verdict(c);
    if (rc) return rc;
    uint32_t flags = c.verdict[0];
    // pending: a sequence whose records were made for another entry state than the one the sequence before it
    // now ends in (k_group_totals).  Its states may all be right, so that the write pass finds nothing, while the
    // counts and DC sums of its first records are not.
    bool pending = c.verdict[2] != 0u;
    // A broken chain (a write lane that did not end in the recorded state) with more than one sequence, or an open
    // boundary, means that the boundaries need more rounds; a broken chain with all boundaries settled is a
    // corrupt stream, and no round will mend it.
    if (pending && c.pl.bnds && c.rounds < c.max_rounds) {
        while (pending && c.rounds < c.max_rounds) {
            ++c.redo;
            hipLaunchKernelGGL(k_clear_status, dim3(1), dim3(64), 0, c.stream, (Status*)(c.ws + c.pl.h.off_status));
            if ((rc = launch_scan(c)) || (rc = launch_report(c, false)) || (rc = wait_verdict(c))) return rc;
            pending = c.verdict[2] != 0u;
        }
        const bool open = pending;
        if ((rc = launch_write(c)) || (rc = launch_report(c, c.want_pixels)) || (rc = wait_verdict(c))) return rc;
        flags = c.verdict[0];
        if (open) flags |= kStMismatch;  // out of rounds: the result is not to be trusted
    } else if (pending && c.pl.bnds) {
        flags |= kStMismatch;
    }
    if (report) {
        memset(report, 0, sizeof *report);
        report->subseq_bits = c.pl.L;
        report->n_subseq = c.pl.nsub_total;
        report->n_sequences = c.pl.seqs;
        report->inter_rounds = c.rounds;
        report->redo = c.redo;
        report->device_flags = flags;
        for (int k = 0; k < JPGD_N_KERNELS; ++k) report->launches[k] = c.launches[k];
        for (const Timed& t : c.timed) {
            float ms = 0.f;
            (void)hipEventSynchronize(c.timers[t.ev + 1]);  // the pixel kernel may still be running
            if (hipEventElapsedTime(&ms, c.timers[t.ev], c.timers[t.ev + 1]) == hipSuccess)
                report->kernel_ms[t.kernel] += ms;
        }
    }
    return flags ? JPGD_E_CORRUPT : JPGD_OK;
}
#undef LAUNCH

bool bad_pointers(int n, const jpgd_info* infos, const uint8_t* d_scans, const uint64_t* scan_offsets, int16_t* d_coef,
                  const uint64_t* coef_offsets, uint8_t* d_pixels, const uint64_t* pixel_offsets) {
    if (!infos || n < 1 || !d_scans || !scan_offsets || !d_coef || !coef_offsets) return true;
    if (d_pixels && !pixel_offsets) return true;
    return ((uintptr_t)d_scans & 15u) || ((uintptr_t)d_coef & 15u);
}

// A call that failed after its first launch: kernels already queued may still read the slot's pinned buffer, so
// the stream is drained before the slot goes back.
void abandon_call(Call* c) {
    if (c->launched) (void)hipStreamSynchronize(c->stream);
    c->launched = false;
    call_release(c);
}

// ---- device memory for the entry point that allocates nothing ------------------------------------------
// A workspace of fixed size inside the library's own image, one copy per GPU.  The name is only a handle on the
// host: the address kernels can use is asked from the runtime, once per device, and kept.
static __device__ __align__(256) uint8_t scratch[kStaticWsBytes];

struct DeviceSetup {
    bool ready = false;
    uint8_t* scratch_ptr = nullptr;  // device address of `scratch` on this device
    Call* call = nullptr;            // the fixed slot of jpgd_decode_static on this device
    std::mutex in_use;               // calls through the fixed slot take turns
};
DeviceSetup g_dev[kMaxDevices];

}  // namespace

extern "C" size_t jpgd_workspace_bytes(const jpgd_info* infos, int n_images, const jpgd_config* cfg) {
    Plan pl;
    if (make_plan(infos, n_images, cfg, pl) != JPGD_OK) return 0;
    return pl.h.total_bytes;
}

extern "C" int jpgd_decode_batch_async(int n, const jpgd_info* infos, const uint8_t* d_scans, const uint64_t* scan_offsets,
                                       int16_t* d_coef, const uint64_t* coef_offsets, uint8_t* d_pixels,
                                       const uint64_t* pixel_offsets, void* d_workspace, size_t workspace_bytes,
                                       const jpgd_config* cfg, void* stream, jpgd_call** call) {
    if (!call) return JPGD_E_ARG;
    *call = nullptr;
    if (bad_pointers(n, infos, d_scans, scan_offsets, d_coef, coef_offsets, d_pixels, pixel_offsets) || !d_workspace)
        return JPGD_E_ARG;
    if ((uintptr_t)d_workspace & 255u) return JPGD_E_WORKSPACE;
    Call* c = nullptr;
    int rc = call_acquire(&c);
    if (rc) return rc;
    c->launched = false;
    rc = enqueue_call(*c, n, infos, d_scans, scan_offsets, d_coef, coef_offsets, d_pixels, pixel_offsets, d_workspace,
                      workspace_bytes, cfg, (hipStream_t)stream);
    if (rc) {
        abandon_call(c);
        return rc;
    }
    *call = c;
    return JPGD_OK;
}

extern "C" int jpgd_wait(jpgd_call* call, jpgd_report* report) {
    if (!call) return JPGD_E_ARG;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        bool known = false;
        for (Call* c : g_calls) known = known || c == call;
        if (!known || !call->busy || call->fixed) return JPGD_E_ARG;
    }
    const int rc = finish_call(*call, report);
    if (rc == JPGD_E_HIP) abandon_call(call);
    else call_release(call);
    return rc;
}

extern "C" int jpgd_decode_batch(int n, const jpgd_info* infos, const uint8_t* d_scans, const uint64_t* scan_offsets,
                                 int16_t* d_coef, const uint64_t* coef_offsets, uint8_t* d_pixels,
                                 const uint64_t* pixel_offsets, void* d_workspace, size_t workspace_bytes,
                                 const jpgd_config* cfg, void* stream, jpgd_report* report) {
    jpgd_call* call = nullptr;
    const int rc = jpgd_decode_batch_async(n, infos, d_scans, scan_offsets, d_coef, coef_offsets, d_pixels, pixel_offsets,
                                           d_workspace, workspace_bytes, cfg, stream, &call);
    if (rc) return rc;
    return jpgd_wait(call, report);
}

extern "C" int jpgd_decode(const jpgd_info* info, const uint8_t* d_scan, int16_t* d_coef, uint8_t* d_pixels,
                           void* d_workspace, size_t workspace_bytes, const jpgd_config* cfg, void* stream,
                           jpgd_report* report) {
    const uint64_t zero = 0;
    return jpgd_decode_batch(1, info, d_scan, &zero, d_coef, &zero, d_pixels, &zero, d_workspace, workspace_bytes, cfg,
                             stream, report);
}

extern "C" int jpgd_init(void) {
    int dev = 0;
    HIP_OK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return JPGD_E_ARG;
    DeviceSetup& D = g_dev[dev];
    std::lock_guard<std::mutex> turn(D.in_use);
    if (D.ready) return JPGD_OK;
    uint8_t* ptr = nullptr;
    HIP_OK(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || ((uintptr_t)ptr & 255u)) return JPGD_E_HIP;
    Call* c = new Call();
    c->device = dev;
    int rc = call_reserve(*c, kStaticStageBytes);
    if (rc) {
        delete c;
        return rc;
    }
    c->fixed = true;
    // Dynamic LDS of the kernels as the fixed-size entry point may need it (one image, any subsequence size): asked for
    // here, so that the entry point itself changes no attribute of a function.
    const void* const sync_kernels[4] = {(const void*)k_sync_intra<true, false>, (const void*)k_sync_intra<false, false>,
                                         (const void*)k_sync_intra<true, true>, (const void*)k_sync_intra<false, true>};
    for (int v = 0; v < 4; ++v)
        if ((rc = grant_lds(dev, v, sync_kernels[v], lds_sync_bytes(2048u, kMaxSlots, kMaxPairs, v >= 2)))) break;
    if (!rc) rc = grant_lds(dev, 6, (const void*)k_sync_head<true, false>, lds_sync_bytes(2048u, kMaxSlots, kMaxPairs, false));
    if (!rc) rc = grant_lds(dev, 4, (const void*)k_write<true>, lds_write_bytes(2048u, kMaxSlots, true));
    if (!rc) rc = grant_lds(dev, 5, (const void*)k_write<false>, lds_write_bytes(2048u, kMaxSlots, true));
    if (!rc) rc = grant_lds(dev, 8, (const void*)k_sync_inter, (size_t)kMaxSlots * kLutEntries * 2);
    if (rc) return rc;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        g_calls.push_back(c);
    }
    D.scratch_ptr = ptr;
    D.call = c;
    D.ready = true;
    return JPGD_OK;
}

extern "C" size_t jpgd_static_workspace_bytes(void) { return kStaticWsBytes; }

extern "C" int jpgd_decode_static(const jpgd_info* info, const uint8_t* d_scan, int16_t* d_coef, uint8_t* d_pixels,
                                  const jpgd_config* cfg, void* stream, jpgd_report* report) {
    const uint64_t zero = 0;
    if (bad_pointers(1, info, d_scan, &zero, d_coef, &zero, d_pixels, &zero)) return JPGD_E_ARG;
    if (cfg && cfg->timing_mask) return JPGD_E_ARG;  // events would have to be created
    int dev = 0;
    HIP_OK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return JPGD_E_ARG;
    DeviceSetup& D = g_dev[dev];
    std::lock_guard<std::mutex> turn(D.in_use);  // one call at a time: they all use the device's one array
    if (!D.ready) {
        fprintf(stderr, "jpgd: jpgd_decode_static needs jpgd_init() on this device first\n");
        return JPGD_E_ARG;
    }
    {
        // sizes beyond the fixed workspace or the fixed parameter buffer are refused before anything is launched
        Plan pl;
        const int rc = make_plan(info, 1, cfg, pl);
        if (rc) return rc;
        if (pl.h.total_bytes > kStaticWsBytes || pl.h.upload_bytes + 16 > D.call->cap) {
            fprintf(stderr, "jpgd: jpgd_decode_static: this image needs %zu bytes of workspace, the built-in one has %zu\n",
                    (size_t)pl.h.total_bytes, kStaticWsBytes);
            return JPGD_E_WORKSPACE;
        }
    }
    Call& c = *D.call;
    c.busy = true;
    c.launched = false;
    int rc = enqueue_call(c, 1, info, d_scan, &zero, d_coef, &zero, d_pixels, &zero, D.scratch_ptr, kStaticWsBytes, cfg,
                          (hipStream_t)stream);
    if (!rc) rc = finish_call(c, report);
    if (rc != JPGD_OK && rc != JPGD_E_CORRUPT && c.launched) (void)hipStreamSynchronize(c.stream);
    c.busy = false;
    return rc;
}

extern "C" int jpgd_read_sync_info(const void* d_workspace, int image, uint32_t capacity, uint32_t* n_subseq,
                                   uint64_t* p, uint32_t* u, uint32_t* z, uint32_t* units, int32_t* dcsum,
                                   void* stream_v) {
    if (!d_workspace || image < 0 || !n_subseq || !p || !u || !z || !units || !dcsum) return JPGD_E_ARG;
    hipStream_t stream = (hipStream_t)stream_v;
    const uint8_t* ws = (const uint8_t*)d_workspace;
    WsHeader h;
    HIP_OK(hipMemcpyAsync(&h, ws, sizeof h, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    if (h.magic != kMagic || (uint32_t)image >= h.nimg) return JPGD_E_ARG;
    ImgDesc d;
    ImgState st;
    HIP_OK(hipMemcpyAsync(&d, ws + h.off_img + sizeof(ImgDesc) * (size_t)image, sizeof d, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(&st, ws + h.off_state + sizeof(ImgState) * (size_t)image, sizeof st, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    *n_subseq = st.nsub;
    if (st.nsub > capacity) return JPGD_E_ARG;
    std::vector<SInfo> rec(st.nsub);
    if (st.nsub) {
        HIP_OK(hipMemcpyAsync(rec.data(), ws + h.off_sinfo + sizeof(SInfo) * (size_t)d.sub0, sizeof(SInfo) * (size_t)st.nsub,
                              hipMemcpyDeviceToHost, stream));
        HIP_OK(hipStreamSynchronize(stream));
    }
    for (uint32_t i = 0; i < st.nsub; ++i) {
        p[i] = ((uint64_t)(i + 1) << h.logL) + state_prel(rec[i].x);
        z[i] = state_z(rec[i].x);
        u[i] = state_u(rec[i].x);
        units[i] = rec[i].y;
        dcsum[3 * i + 0] = (int16_t)(rec[i].z & 0xFFFFu);
        dcsum[3 * i + 1] = (int16_t)(rec[i].z >> 16);
        dcsum[3 * i + 2] = (int16_t)(rec[i].w & 0xFFFFu);
    }
    return JPGD_OK;
}

extern "C" int jpgd_unstuff(const uint8_t* d_in, size_t n, uint8_t* d_out, size_t* out_len, void* d_workspace,
                            size_t workspace_bytes, void* stream_v) {
    if (!d_in || !d_out || !out_len || !d_workspace || n < 1 || n >= (1ull << 28)) return JPGD_E_ARG;
    if (((uintptr_t)d_in & 15u) || ((uintptr_t)d_out & 255u) || ((uintptr_t)d_workspace & 255u)) return JPGD_E_ARG;
    const uint32_t tiles = (uint32_t)((n + kUnstuffTile - 1) / kUnstuffTile);
    const size_t off_state = 0, off_img = 256, off_tiles = up256(256 + sizeof(ImgDesc));
    const size_t need = up256(off_tiles + (size_t)tiles * 4);
    if (workspace_bytes < need) return JPGD_E_WORKSPACE;
    hipStream_t stream = (hipStream_t)stream_v;
    Call* c = nullptr;
    int rc = call_acquire(&c);
    if (rc) return rc;
    struct Release {
        Call* c;
        hipStream_t s;
        ~Release() {
            (void)hipStreamSynchronize(s);
            call_release(c);
        }
    } release{c, stream};
    rc = call_reserve(*c, off_tiles);
    if (rc) return rc;
    uint8_t* up = c->buf;
    memset(up, 0, off_tiles);
    ImgDesc d;
    memset(&d, 0, sizeof d);
    d.scan_bytes = (uint32_t)n;
    d.ntiles = tiles;
    memcpy(up + off_img, &d, sizeof d);
    uint8_t* ws = (uint8_t*)d_workspace;
    HIP_OK(hipMemcpyAsync(ws, up, off_tiles, hipMemcpyHostToDevice, stream));
    Params P;
    memset(&P, 0, sizeof P);
    P.img = (const ImgDesc*)(ws + off_img);
    P.st = (ImgState*)(ws + off_state);
    P.scans = d_in;
    P.stream = d_out;
    P.tile_cnt = (uint32_t*)(ws + off_tiles);
    P.nimg = 1;
    P.img0 = d;
    P.logL = 10;
    hipLaunchKernelGGL(k_unstuff_count, dim3(tiles), dim3(kWG), 0, stream, P);
    if (tiles > (uint32_t)kWG) hipLaunchKernelGGL(k_unstuff_scan, dim3(1), dim3(kWG), 0, stream, P);
    hipLaunchKernelGGL(k_unstuff_scatter, dim3(tiles), dim3(kWG), 0, stream, P);
    HIP_OK(hipGetLastError());
    HIP_OK(hipMemcpyAsync(c->verdict, ws + off_state, sizeof(ImgState), hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    *out_len = c->verdict[0];
    return JPGD_OK;
}
