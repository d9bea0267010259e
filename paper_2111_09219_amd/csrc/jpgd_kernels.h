// gfx950 kernels of the decoder.  Included once, by jpgd.hip.
//
// Launch geometry: every kernel runs kWG = 256 lanes (four wave64) per workgroup, except the
// inter-sequence kernel (one wave64).  A workgroup finds its image by bisection over the per-image
// first-workgroup fields of ImgDesc, so one launch covers a whole batch.
#pragma once
#include <hip/hip_runtime.h>

#include "jpgd_common.h"
#include "jpgd_idct.h"
#include "jpgd_lane.h"

namespace jpgd {

struct Params {
    const ImgDesc* img;
    ImgState* st;
    Status* status;
    const uint8_t* scans;
    uint8_t* stream;        // unstuffed streams, image i at img[i].stream_off
    uint32_t* tile_cnt;     // per unstuff tile: bytes removed in it (low half) and restart markers met in it (high
                            // half), then (in place, images of more than 256 tiles) bytes removed before it
    SInfo* sinfo;
    int4* grp_tot;          // per group of kWG subsequences: (units, dc0, dc1, dc2) totals
    int4* grp_pref;         // exclusive prefix of grp_tot inside the image
    uint32_t* bmap;         // interval-start bitmaps of images with restart intervals (ImgDesc::bmap_off)
    uint32_t* seq_rec;      // split synchronisation: per sequence 4 x kWG words, the records of all its lanes after their
                            // own subsequence (state, units, DC sums), handed from the first kernel to the second
    uint32_t* warm_x;       // per sequence: the state at its first subsequence's start that its records continue
                            // (packed like SInfo::x; 0xFFFFFFFF = none)
    const uint16_t* luts;
    const uint16_t* qts;
    int16_t* coef;
    uint8_t* pixels;
    uint32_t nimg;
    uint32_t logL;          // log2 of the subsequence size in bits
    uint32_t overlap;       // H: warm-up lanes in front of each sequence
    uint32_t seq_len;       // kWG - H: subsequences a sequence owns
    uint32_t lut_slots;     // max tables of any image (sizes the LDS copy)
    uint32_t pair_slots;    // max AC tables of any image (sizes the LDS copy of their pair bytes)
    uint32_t planar;        // pixel kernel: component planes (no upsampling, no colour conversion) instead of RGB
    uint32_t scale_log2;    // pixel kernel: output at 1/2^scale_log2 of the size (0..3)
    uint32_t handoff;       // intra-sequence kernel, split in two: chains left at which the first hands over (at most 64)
    uint32_t coop_max;      // intra-sequence kernel: with at most this many chains left, one wavefront per chain
    uint32_t sync_waves;    // wavefronts per workgroup of that kernel: kWG / 64 that hold the lanes, the rest only take chains
    // A call with one image has the last up_wgs workgroups of k_unstuff_count copy the call's parameter block
    // (up_n16 16-byte words) from pinned host memory into the workspace: that kernel does not need the block, all
    // later ones do, and a kernel of its own for the copy would cost a dispatch.  up_wgs = 0: nothing to copy.
    const uint4* up_src;
    uint4* up_dst;
    uint32_t up_n16;
    uint32_t up_wgs;
    // pixel kernel: where its first lane reports the outcome of the write kernel before anything else (pinned host
    // memory: flags, inter_changed, pending, .., ticket in word 15; null = somebody else reports) and this call's ticket
    uint32_t* verdict;
    uint32_t ticket;
    // A call with one image carries its descriptor in the kernel arguments: every workgroup of every kernel
    // starts by reading the descriptor, and when all of them ask memory for the same freshly written line
    // that read alone was measured at 1 to 11 microseconds per kernel.
    ImgDesc img0;
};

// A workgroup's image descriptor.  It is the same for every lane, but the compiler cannot see that (it merges
// the two sources into one load through a generic pointer and takes the result for lane-dependent), so what
// follows from it sits in vector registers and branches on it are taken with execution masks.
__device__ __forceinline__ ImgDesc image_desc(const Params& P, uint32_t ii) {
    if (P.nimg == 1u) return P.img0;
    return P.img[ii];
}

// The same with every word passed through readfirstlane: the descriptor and what follows from it stay in scalar
// registers and branches on it are scalar branches.  Measured per kernel: pixels 9 %, write 2 % and
// unstuff_count 8 % faster with it; the two synchronisation kernels 2 to 4 % slower (their lane decoder is short
// of scalar registers, not of vector ones), so they keep the plain form.
__device__ __forceinline__ ImgDesc image_desc_uniform(const Params& P, uint32_t ii) {
    ImgDesc d = image_desc(P, ii);
    static_assert(sizeof(ImgDesc) % 4u == 0u, "descriptor is copied word by word");
    uint32_t w[sizeof(ImgDesc) / 4u];
    __builtin_memcpy(w, &d, sizeof d);
#pragma unroll
    for (uint32_t i = 0; i < sizeof(ImgDesc) / 4u; ++i) w[i] = __builtin_amdgcn_readfirstlane(w[i]);
    __builtin_memcpy(&d, w, sizeof d);
    return d;
}

// ---- small helpers ------------------------------------------------------------------------------

template <class F>
__device__ __forceinline__ uint32_t find_image(const Params& P, uint32_t wg, F first_wg) {
    uint32_t lo = 0, hi = P.nimg;  // last image whose first workgroup is <= wg
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (first_wg(P.img[mid]) <= wg) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = __shfl_up(v, d, 64);
        if (lane >= (uint32_t)d) v += o;
    }
    return v;
}

// exclusive prefix of v over the 256 lanes of the workgroup; *total gets the sum.  scratch: 8 words of LDS.
__device__ __forceinline__ uint32_t wg_excl_scan(uint32_t v, uint32_t* scratch, uint32_t* total) {
    uint32_t inc = wave_incl_scan(v);
    uint32_t wave = threadIdx.x >> 6;
    __syncthreads();  // scratch may still be read from a previous use
    if ((threadIdx.x & 63u) == 63u) scratch[wave] = inc;
    __syncthreads();
    uint32_t w0 = scratch[0], w1 = scratch[1], w2 = scratch[2], w3 = scratch[3];
    uint32_t before = wave == 0 ? 0u : wave == 1 ? w0 : wave == 2 ? w0 + w1 : w0 + w1 + w2;
    *total = w0 + w1 + w2 + w3;
    return before + inc - v;
}

// What the scan over s_info carries (paper, Algorithm 1: exclusive prefix sum on s_info.n; Section 4.2: prefix
// sum of the DC differences): data units, and the DC sums of the three components.  With restart intervals
// the DC sums are a segmented sum: a record whose subsequence holds the first symbol of an interval (flag)
// starts them afresh.  join(a, b) = a followed by b; it is associative, so the usual scans apply.
// (the sums are kept unsigned: only their low 16 bits are used and they may wrap on the way)
struct Seg {
    uint32_t units, flag;
    uint32_t d0, d1, d2;
};
__device__ __forceinline__ Seg seg_zero() { return Seg{0u, 0u, 0u, 0u, 0u}; }
__device__ __forceinline__ Seg seg_join(const Seg& a, const Seg& b) {
    Seg r;
    r.units = a.units + b.units;
    r.flag = a.flag | b.flag;
    r.d0 = b.flag ? b.d0 : a.d0 + b.d0;
    r.d1 = b.flag ? b.d1 : a.d1 + b.d1;
    r.d2 = b.flag ? b.d2 : a.d2 + b.d2;
    return r;
}
__device__ __forceinline__ uint32_t sx16(uint32_t v) { return (uint32_t)(int32_t)(int16_t)(v & 0xFFFFu); }
__device__ __forceinline__ Seg seg_of_record(const SInfo& r) {
    return Seg{rec_units(r.y), rec_restarted(r.y), sx16(r.z), sx16(r.z >> 16), sx16(r.w)};
}
// group totals travel as int4: units with the flag in bit 31, then the three sums
__device__ __forceinline__ int4 seg_pack(const Seg& s) { return make_int4((int)(s.units | (s.flag << 31)), (int)s.d0, (int)s.d1, (int)s.d2); }
__device__ __forceinline__ Seg seg_unpack(const int4& v) {
    return Seg{(uint32_t)v.x & 0x7FFFFFFFu, (uint32_t)v.x >> 31, (uint32_t)v.y, (uint32_t)v.z, (uint32_t)v.w};
}
__device__ __forceinline__ Seg seg_shfl_up(const Seg& v, int d) {
    Seg o;
    o.units = __shfl_up(v.units, d, 64); o.flag = __shfl_up(v.flag, d, 64);
    o.d0 = __shfl_up(v.d0, d, 64); o.d1 = __shfl_up(v.d1, d, 64); o.d2 = __shfl_up(v.d2, d, 64);
    return o;
}

// exclusive scan of v over the 256 lanes of the workgroup under seg_join; *total gets the join of all.
// scratch: 20 words of LDS.
__device__ __forceinline__ Seg wg_excl_segscan(Seg v, uint32_t* scratch, Seg* total) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    Seg inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const Seg o = seg_shfl_up(inc, d);
        if (lane >= (uint32_t)d) inc = seg_join(o, inc);
    }
    __syncthreads();  // scratch may still be read from a previous use
    if (lane == 63u) {
        uint32_t* s5 = scratch + wave * 5u;
        s5[0] = inc.units; s5[1] = inc.flag; s5[2] = inc.d0; s5[3] = inc.d1; s5[4] = inc.d2;
    }
    __syncthreads();
    Seg carry = seg_zero(), all = seg_zero();
#pragma unroll
    for (uint32_t k = 0; k < 4u; ++k) {
        const uint32_t* s5 = scratch + k * 5u;
        const Seg t = Seg{s5[0], s5[1], s5[2], s5[3], s5[4]};
        if (k < wave) carry = seg_join(carry, t);
        all = seg_join(all, t);
    }
    *total = all;
    Seg before = seg_shfl_up(inc, 1);
    if (lane == 0u) before = seg_zero();
    return seg_join(carry, before);
}

__device__ __forceinline__ void stage_luts(const Params& P, const ImgDesc& D, uint16_t* lut_s) {
    const uint32_t n16 = D.nslots * (uint32_t)kLutEntries;       // uint16 count, multiple of 8
    const uint4* src = reinterpret_cast<const uint4*>(P.luts + D.lut_off);
    uint4* dst = reinterpret_cast<uint4*>(lut_s);
    for (uint32_t k = threadIdx.x; k < n16 / 8u; k += blockDim.x) dst[k] = src[k];
}

// pair bytes of the image's AC tables, behind its table slots in memory; pair_of_unit: 8 words of LDS
__device__ __forceinline__ void stage_pairs(const Params& P, const ImgDesc& D, uint8_t* pair_s, uint32_t* pair_of_unit) {
    const uint32_t n16 = (D.nslots - D.ndc) * (uint32_t)(kPairBytes / 16);
    const uint4* src = reinterpret_cast<const uint4*>(P.luts + D.lut_off + (uint32_t)(kMaxSlots * kLutEntries));
    uint4* dst = reinterpret_cast<uint4*>(pair_s);
    for (uint32_t k = threadIdx.x; k < n16; k += blockDim.x) dst[k] = src[k];
    if (threadIdx.x < D.upm)
        pair_of_unit[threadIdx.x] = (((D.sched_ac >> (4u * threadIdx.x)) & 15u) - D.ndc) * (uint32_t)kPairBytes;
}

// rows: 8 entries of LDS, complete after the next barrier
__device__ __forceinline__ Syntax stage_syntax(const ImgDesc& D, UnitRow* rows) {
    if (threadIdx.x < D.upm) rows[threadIdx.x] = make_unit_row(threadIdx.x, D.upm, D.sched_dc, D.sched_ac, D.sched_comp);
    Syntax sx;
    sx.rows = rows;
    sx.upm = D.upm;
    return sx;
}

// LDS copy of a stretch of the stream as big-endian 32-bit words.  No padding: lanes start a power of two
// apart and collide on a bank for their first reads only; after that they advance at their own pace.
__device__ __forceinline__ void stage_stream(const uint8_t* stream_img, uint32_t first_word, uint32_t nwords,
                                             uint32_t* strm) {
    // nwords is a multiple of 4 and first_word*4 a multiple of 16
    const uint4* src = reinterpret_cast<const uint4*>(stream_img + (size_t)first_word * 4u);
    uint4* dst = reinterpret_cast<uint4*>(strm);
    for (uint32_t k = threadIdx.x; k < nwords / 4u; k += blockDim.x) {
        uint4 v = src[k];
        v.x = __builtin_bswap32(v.x); v.y = __builtin_bswap32(v.y);
        v.z = __builtin_bswap32(v.z); v.w = __builtin_bswap32(v.w);
        dst[k] = v;
    }
}

// LDS copy of the part of an image's interval-start bitmap that covers stream words first_word .. +nwords;
// word k of the bitmap is then bm_s[k - (first_word >> 3)]
// Returns the OR of the words this lane copied: most workgroups of a scan with long intervals find no interval
// start at all in their stretch and can run the plain loops.
// With keep == false nothing is stored: the words are only looked at (subsequences of more than kBitmapLdsMaxL bits,
// whose kernels then read the few bitmap words they need from memory; see kBitmapLdsMaxL).
__device__ __forceinline__ uint32_t stage_bitmap(const uint32_t* bmap_img, uint32_t first_word, uint32_t nwords, uint32_t* bm_s,
                                                 bool keep) {
    const uint32_t k0 = first_word >> 3;
    const uint32_t n = ((first_word + nwords + 7u) >> 3) - k0 + 1u;
    uint32_t seen = 0u;
    for (uint32_t k = threadIdx.x; k < n; k += blockDim.x) {
        const uint32_t v = bmap_img[k0 + k];
        if (keep) bm_s[k] = v;
        seen |= v;
    }
    return seen;
}

__device__ __forceinline__ uint32_t pack_dc01(int64_t acc) {
    int32_t d0, d1, d2;
    dc_unpack(acc, d0, d1, d2);
    return ((uint32_t)d0 & 0xFFFFu) | ((uint32_t)d1 << 16);
}
__device__ __forceinline__ uint32_t pack_dc2(int64_t acc) {
    int32_t d0, d1, d2;
    dc_unpack(acc, d0, d1, d2);
    return (uint32_t)d2 & 0xFFFFu;
}

// ---- unstuffing (byte compaction) -----------------------------------------------------------------
// A 0x00 is dropped iff the byte before it is 0xFF: inside entropy-coded data a 0xFF is always followed by
// its stuffed 0x00 or, in a scan with restart intervals, by the second byte of a marker RST0..RST7; both
// bytes of such a marker are dropped too, and the byte that follows it is the first of an interval.  All
// decisions are local (one byte back, one byte ahead).

struct UnstuffLane {
    uint32_t bytes[4];  // 16 input bytes
    uint32_t keep_mask; // bit j set = byte j is kept
    uint32_t mark_mask; // bit j set = byte j is the second byte of a restart marker
    uint32_t nvalid;    // bytes of this lane that exist
};

// pos is a multiple of 16.  A lane that holds any byte loads its whole 16-byte word (the input is readable up
// to the next multiple of 16); bytes past the end are masked out.  No private array is indexed with a variable:
// the compiler would move such an array to LDS and read the dispatch packet for the workgroup's shape, and that
// packet lives in host memory -- measured at 2 to 11 microseconds per wavefront when a whole grid asks at once.
__device__ __forceinline__ UnstuffLane unstuff_load(const uint8_t* scan, uint32_t n, uint32_t pos, bool restart) {
    UnstuffLane r;
    r.nvalid = pos >= n ? 0u : (n - pos < 16u ? n - pos : 16u);
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r.nvalid) v = *reinterpret_cast<const uint4*>(scan + pos);
    r.bytes[0] = v.x; r.bytes[1] = v.y; r.bytes[2] = v.z; r.bytes[3] = v.w;
    uint32_t prev = (pos > 0u && r.nvalid) ? scan[pos - 1u] : 0u;
    const uint32_t after = (restart && pos + 16u < n) ? scan[pos + 16u] : 0u;
    uint32_t mask = 0u, marks = 0u;
#pragma unroll
    for (uint32_t j = 0; j < 16u; ++j) {
        const uint32_t b = (r.bytes[j >> 2] >> (8u * (j & 3u))) & 255u;
        const uint32_t nx = j < 15u ? (r.bytes[(j + 1u) >> 2] >> (8u * ((j + 1u) & 3u))) & 255u : after;
        const bool exists = j < r.nvalid;
        const bool nx_exists = j + 1u < r.nvalid || (j == 15u && pos + 16u < n);
        const bool rst2 = restart && prev == 255u && (b & 0xF8u) == 0xD0u;                // RSTm, second byte
        const bool rst1 = restart && b == 255u && nx_exists && (nx & 0xF8u) == 0xD0u;     // RSTm, first byte
        const bool drop = (b == 0u && prev == 255u) || rst1 || rst2;
        if (exists && !drop) mask |= 1u << j;
        if (exists && rst2) marks |= 1u << j;
        prev = b;
    }
    r.keep_mask = mask;
    r.mark_mask = marks;
    return r;
}

__global__ __launch_bounds__(kWG) void k_unstuff_count(Params P) {
    __shared__ uint32_t scratch[8];
    const uint32_t wg = blockIdx.x;
    if (P.up_wgs && wg >= gridDim.x - P.up_wgs) {  // the copy of the parameter block (one image per call only)
        const uint32_t first = gridDim.x - P.up_wgs;
        for (uint32_t k = (wg - first) * kWG + threadIdx.x; k < P.up_n16; k += P.up_wgs * kWG) P.up_dst[k] = P.up_src[k];
        return;
    }
    const uint32_t ii = find_image(P, wg, [](const ImgDesc& d) { return d.tile0; });
    const ImgDesc D = image_desc_uniform(P, ii);
    const uint32_t lt = wg - D.tile0;
    const uint8_t* scan = P.scans + D.scan_off;
    const uint32_t pos = lt * (uint32_t)kUnstuffTile + threadIdx.x * 16u;
    const bool restart = D.restart != 0u;
    UnstuffLane u = unstuff_load(scan, D.scan_bytes, pos, restart);
    uint32_t removed = u.nvalid - (uint32_t)__popc(u.keep_mask);
    uint32_t total;
    wg_excl_scan(removed, scratch, &total);
    uint32_t marks = 0u;
    if (restart) {
        // this tile's share of the interval-start bitmap is cleared here, the scatter kernel sets the bits;
        // the markers are counted so that the write pass can tell whether all intervals are there
        uint32_t* bm = P.bmap + D.bmap_off + lt * 128u;
        if (threadIdx.x < 128u) bm[threadIdx.x] = 0u;
        if (lt == D.ntiles - 1u && threadIdx.x < 128u) bm[128u + threadIdx.x] = 0u;
        wg_excl_scan((uint32_t)__popc(u.mark_mask), scratch, &marks);
    }
    if (threadIdx.x == 0) P.tile_cnt[wg] = total | (marks << 16);  // at most 4096 and 2048
}

// one workgroup per image: per-tile counts -> bytes removed before each tile; unstuffed length and
// number of subsequences of the image
__global__ __launch_bounds__(kWG) void k_unstuff_scan(Params P) {
    __shared__ uint32_t scratch[8];
    const uint32_t ii = blockIdx.x;
    const ImgDesc D = image_desc_uniform(P, ii);
    if (D.ntiles <= (uint32_t)kWG) return;  // images of up to 256 tiles: the scatter kernel sums the counts itself
    // every lane takes a run of consecutive tiles: sum, one scan over the 256 sums, then the prefixes inside the run
    // (one pair of barriers in all; a loop of 256-tile scans was measured at 0.7 microseconds per step)
    uint32_t* cnt = P.tile_cnt + D.tile0;
    const uint32_t per = (D.ntiles + (uint32_t)kWG - 1u) / (uint32_t)kWG;
    const uint32_t k0 = min(threadIdx.x * per, D.ntiles), k1 = min(k0 + per, D.ntiles);
    uint32_t sum = 0u, msum = 0u;
#pragma unroll 8
    for (uint32_t k = k0; k < k1; ++k) {
        const uint32_t v = cnt[k];
        sum += v & 0xFFFFu;
        msum += v >> 16;
    }
    uint32_t carry, markers;
    wg_excl_scan(msum, scratch, &markers);
    uint32_t ex = wg_excl_scan(sum, scratch, &carry);
#pragma unroll 8
    for (uint32_t k = k0; k < k1; ++k) {
        const uint32_t v = cnt[k] & 0xFFFFu;
        cnt[k] = ex;
        ex += v;
    }
    if (threadIdx.x == 0) {
        uint32_t nbytes = D.scan_bytes - carry;
        P.st[ii].markers = markers;
        P.st[ii].nbytes = nbytes;
        uint32_t L = 1u << P.logL;
        P.st[ii].nsub = (uint32_t)(((uint64_t)nbytes * 8u + L - 1u) >> P.logL);
    }
}

__global__ __launch_bounds__(kWG) void k_unstuff_scatter(Params P) {
    __shared__ uint32_t scratch[8];
    __shared__ __attribute__((aligned(16))) uint8_t buf[kUnstuffTile + 16];
    const uint32_t wg = blockIdx.x;
    const uint32_t ii = find_image(P, wg, [](const ImgDesc& d) { return d.tile0; });
    const ImgDesc D = image_desc_uniform(P, ii);
    const uint32_t lt = wg - D.tile0;
    const uint8_t* scan = P.scans + D.scan_off;
    uint8_t* out = P.stream + D.stream_off;
    const uint32_t pos = lt * (uint32_t)kUnstuffTile + threadIdx.x * 16u;
    UnstuffLane u = unstuff_load(scan, D.scan_bytes, pos, D.restart != 0u);
    uint32_t kept = (uint32_t)__popc(u.keep_mask);
    uint32_t T;
    uint32_t off = wg_excl_scan(kept, scratch, &T);
    const uint32_t lane_off = off;
#pragma unroll
    for (uint32_t j = 0; j < 16u; ++j)
        if (u.keep_mask & (1u << j)) buf[off++] = (uint8_t)(u.bytes[j >> 2] >> (8u * (j & 3u)));
    __syncthreads();
    // bytes removed before this tile: from the scan kernel, or, for images of up to 256 tiles, summed here
    uint32_t before, nbytes;
    if (D.ntiles <= (uint32_t)kWG) {
        const uint32_t raw = threadIdx.x < D.ntiles ? P.tile_cnt[D.tile0 + threadIdx.x] : 0u;
        const uint32_t v = raw & 0xFFFFu;
        uint32_t all, markers = 0u;
        wg_excl_scan(v, scratch, &all);
        wg_excl_scan(threadIdx.x < lt ? v : 0u, scratch, &before);
        if (D.restart != 0u && lt == 0u) wg_excl_scan(raw >> 16, scratch, &markers);
        nbytes = D.scan_bytes - all;
        if (lt == 0u && threadIdx.x == 0u) {
            P.st[ii].markers = markers;
            P.st[ii].nbytes = nbytes;
            P.st[ii].nsub = (uint32_t)(((uint64_t)nbytes * 8u + (1u << P.logL) - 1u) >> P.logL);
        }
    } else {
        before = P.tile_cnt[wg];
        nbytes = P.st[ii].nbytes;
    }
    // output position of this tile's first kept byte
    const uint32_t o = lt * (uint32_t)kUnstuffTile - before;
    const uint32_t a = o & 3u;
    const uint32_t nd = (a + T + 3u) >> 2;
    uint32_t* out32 = reinterpret_cast<uint32_t*>(out + (o - a));
    for (uint32_t d = threadIdx.x; d < nd; d += kWG) {
        int32_t s0 = (int32_t)(4u * d) - (int32_t)a;
        if (s0 >= 0 && (uint32_t)s0 + 4u <= T) {
            uint32_t v = (uint32_t)buf[s0] | ((uint32_t)buf[s0 + 1] << 8) | ((uint32_t)buf[s0 + 2] << 16) |
                         ((uint32_t)buf[s0 + 3] << 24);
            out32[d] = v;
        } else {
            for (int32_t b = 0; b < 4; ++b) {
                int32_t s = s0 + b;
                if (s >= 0 && (uint32_t)s < T) out[o - a + 4u * d + (uint32_t)b] = buf[s];
            }
        }
    }
    // the byte after a restart marker starts an interval: its position in the output goes into the bitmap
    if (u.mark_mask) {
        uint32_t* bm = P.bmap + D.bmap_off;
        for (uint32_t m = u.mark_mask; m; m &= m - 1u) {
            const uint32_t j = (uint32_t)__ffs((int)m) - 1u;
            const uint32_t at = o + lane_off + (uint32_t)__popc(u.keep_mask & ((1u << j) - 1u));
            atomicOr(&bm[at >> 5], 1u << (at & 31u));
        }
    }
    // the last tile clears what lanes may read past the end: one subsequence plus 64 bytes
    if (lt == D.ntiles - 1u) {
        const uint32_t clear = (1u << (P.logL - 3u)) + 64u;
        for (uint32_t k = threadIdx.x; k < clear; k += kWG) out[nbytes + k] = 0u;
    }
}

// ---- one chain decoded by a whole wavefront -----------------------------------------------------------
// The last overflow rounds of a sequence have a handful of chains left, and a lane that decodes one symbol
// after the other spends some fifty dependent instructions on each.  So when few chains remain, each goes to a
// wavefront of its own: lane j looks up the symbol that WOULD start j bits after the chain's position, in every
// table of the image at once, and the chain is then followed through those 64 answers with scalar code (a
// readlane and a few scalar operations per symbol) until it leaves the 64-bit window.  The synchronisation pass
// only needs (p, u, z), the count of completed units and the DC sums, so a symbol's value bits matter only for
// DC symbols.  Results are those of decode_span_sync, symbol by symbol.

// lane i < upm describes data unit i of the MCU: slot of its AC table (bits 0-2), slot of the DC table of the
// unit that follows (3-5), index of that unit (6-9), bit offset of its component's field in the DC sums (10-14)
__device__ __forceinline__ uint32_t coop_unit_word(const Syntax& sx, uint32_t lane) {
    if (lane >= sx.upm) return 0u;
    const UnitRow r = sx.rows[lane];
    return (r.tb_ac / (uint32_t)kLutEntries) | ((r.tb_dc_next / (uint32_t)kLutEntries) << 3) | (r.next << 6) |
           (((uint32_t)__ffs((int)r.dcmul) - 1u) << 10);
}

// second-level entry of a codeword longer than the first-level index, asked for by the whole wavefront at once
template <class LutPtr>
__device__ __forceinline__ uint32_t coop_resolve(LutPtr lut, uint32_t slot, uint32_t e, uint32_t peek) {
    const uint32_t nb2 = lut_esc_bits(e);
    const uint32_t at = slot * (uint32_t)kLutEntries + (uint32_t)kLutL1 + lut_esc_offset(e) +
                        ((peek >> (32 - kLutK - nb2)) & ((1u << nb2) - 1u));
    return __builtin_amdgcn_readfirstlane((uint32_t)lut[at]);
}

// the same for every lane's own entry and bits
template <class LutPtr>
__device__ __forceinline__ uint32_t coop_resolve_lane(LutPtr lut, uint32_t slot, uint32_t e, uint32_t peek) {
    const uint32_t nb2 = lut_esc_bits(e);
    return lut[slot * (uint32_t)kLutEntries + (uint32_t)kLutL1 + lut_esc_offset(e) +
               ((peek >> (32 - kLutK - nb2)) & ((1u << nb2) - 1u))];
}

// A table entry as the walk adds it to its packed state (coop_span_sync): bits taken (at least one) in bits 0..4
// and zig-zag slots covered in bits 9..14; for a first-level escape nothing but bit 16, which stops the walk.
constexpr int kCoopUnroll = 8;
__device__ __forceinline__ uint32_t coop_step(uint32_t e) {
    return (e & 0x8000u) ? 0x10000u : ((e & 0x7E00u) | max(e & 31u, 1u));
}

// What the lanes know about one window of 64 bit positions: lane j holds the 32 bits that start at position j and
// the first-level entry of each table for them (a table the image does not have is asked as the last one it has).
struct CoopWindow {
    uint32_t peek, e0, e1, e2, e3;
};

// The window that starts at bit ws (a multiple of 64).  The wavefront keeps 64 consecutive stream words, one per
// lane, from word w0 on, and reloads them when a window needs words beyond them (org_word: stream word with cursor
// 0 of `fetch`; cursors from nwords on are not read).  The table reads are only issued here.
template <class Fetch, class LutPtr>
__device__ __forceinline__ CoopWindow coop_window(uint32_t ws, uint32_t& w0, uint32_t& held, bool& have, uint32_t org_word,
                                                  uint32_t nwords, uint32_t nslots, uint32_t lane, Fetch fetch, LutPtr lut) {
    uint32_t wb = (ws >> 5) - w0;
    if (!have || wb + 2u > 63u) {
        w0 = ws >> 5;
        const uint32_t c = w0 - org_word + lane;
        held = c < nwords ? fetch(c) : 0u;
        wb = 0u;
        have = true;
    }
    const uint32_t s0 = __builtin_amdgcn_readlane(held, wb), s1 = __builtin_amdgcn_readlane(held, wb + 1u);
    const uint32_t s2 = __builtin_amdgcn_readlane(held, wb + 2u);
    const uint32_t hi = lane < 32u ? s0 : s1, lo = lane < 32u ? s1 : s2;
    CoopWindow w;
    w.peek = (uint32_t)(((((uint64_t)hi << 32) | (uint64_t)lo) << (lane & 31u)) >> 32);
    const uint32_t idx = w.peek >> (32 - kLutK);
    w.e0 = lut[idx];
    w.e1 = lut[min(1u, nslots - 1u) * (uint32_t)kLutEntries + idx];
    w.e2 = lut[min(2u, nslots - 1u) * (uint32_t)kLutEntries + idx];
    w.e3 = lut[min(3u, nslots - 1u) * (uint32_t)kLutEntries + idx];
    return w;
}

// p, u, z: wave-uniform state of the chain, advanced until p >= limit (limit a multiple of 64).  org_word, nwords:
// see coop_window.  1 <= nslots <= 4 tables.
// The windows lie on a 64-bit grid of the stream (a subsequence is a whole number of them, and a chain enters a
// subsequence at most 31 bits behind its start, so no window is wasted): the window after the current one is known
// before the chain has been followed through this one, and its table reads are issued first and answered
// meanwhile.  Escapes are followed up in the walk, where only those on the chain matter.
template <class Fetch, class LutPtr>
__device__ __forceinline__ void coop_span_sync(uint32_t& p_io, uint32_t& u_io, uint32_t& z_io, uint32_t& nb_out,
                                               int64_t& dc_out, uint32_t limit, uint32_t org_word, uint32_t nwords,
                                               uint32_t unit_word, uint32_t upm, uint32_t nslots, Fetch fetch,
                                               LutPtr lut) {
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t p = __builtin_amdgcn_readfirstlane(p_io);
    uint32_t u = __builtin_amdgcn_readfirstlane(u_io);
    uint32_t z = __builtin_amdgcn_readfirstlane(z_io);
    uint32_t nb = 0u;
    int64_t dc = 0;
    uint32_t cur = __builtin_amdgcn_readlane(unit_word, u);
    // slots of the current unit's AC table and of the table of the DC symbol that starts it
    uint32_t ac_slot = cur & 7u;
    uint32_t dc_slot = (__builtin_amdgcn_readlane(unit_word, u == 0u ? upm - 1u : u - 1u) >> 3) & 7u;
    uint32_t w0 = 0u, held = 0u;
    bool have = false;
    if (p < limit) {
        uint32_t ws = p & ~63u;
        // S = window position j (bits 0..6, at most 63 + 31) and zig-zag index z (bits 9..15, at most 63 + 63);
        // adding a symbol's step advances both.  Bit 6 set: the window is behind us; bit 15: the data unit is
        // complete; bit 16: the entry was an escape and nothing has been advanced.
        uint32_t S = (p - ws) | (z << 9);
        CoopWindow nxt = coop_window(ws, w0, held, have, org_word, nwords, nslots, lane, fetch, lut);
        // (Without this the compiler merges these reads with the ones inside the loop into reads at the top of the
        // loop, where every window would wait for them.)
        asm volatile("" : "+v"(nxt.e0), "+v"(nxt.e1), "+v"(nxt.e2), "+v"(nxt.e3));
        for (;;) {
            const uint32_t peek = nxt.peek;
            const uint32_t e01 = nxt.e0 | (nxt.e1 << 16), e23 = nxt.e2 | (nxt.e3 << 16);
            const bool more = ws + 64u < limit;
            if (more) nxt = coop_window(ws + 64u, w0, held, have, org_word, nwords, nslots, lane, fetch, lut);
            uint32_t acv = ((ac_slot & 2u) ? e23 : e01) >> ((ac_slot & 1u) << 4);  // the AC entry in the low 16 bits
            uint32_t acs = coop_step(acv);
            for (;;) {
                if ((S >> 9) == 0u) {  // DC symbol (z = 0, so S is j)
                    const uint32_t pair = __builtin_amdgcn_readlane((dc_slot & 2u) ? e23 : e01, S);
                    const uint32_t pk = __builtin_amdgcn_readlane(peek, S);
                    uint32_t r = pair >> ((dc_slot & 1u) << 4);
                    if (r & 0x8000u) r = coop_resolve(lut, dc_slot, r, pk);
                    const int32_t v = symbol_value(pk, lut_total(r), lut_size(r));
                    dc += (int64_t)v * (int64_t)(1u << ((cur >> 10) & 31u));
                    S += coop_step(r);  // z becomes 1, or stays 0 where no codeword starts
                    if (S & 0x40u) break;
                    if ((S >> 9) == 0u) continue;
                }
                // AC symbols up to the end of the unit or of the window.  A taken branch costs a lone wavefront far
                // more than the three other instructions of a step, so the steps come eight in a row with one exit
                // test each, and everything unusual leaves through that exit.
                for (;;) {
                    bool out = false;
#pragma unroll
                    for (int k = 0; k < kCoopUnroll; ++k) {
                        S += __builtin_amdgcn_readlane(acs, S & 63u);
                        if (__builtin_expect((S & 0x18040u) != 0u, 0)) {
                            out = true;
                            break;
                        }
                    }
                    if (!out) continue;
                    if (S & 0x10000u) {
                        // The codeword at this position is longer than the first-level index.  Every lane whose
                        // entry of this table is an escape follows it up now, at once: where codewords are long
                        // (large coefficients) a window holds several on the chain, and one look-up by all lanes
                        // costs less than one by the chain alone.  The step is then taken again.
                        S &= 0xFFFFu;
                        if (acv & 0x8000u) acv = coop_resolve_lane(lut, ac_slot, acv, peek);
                        acs = coop_step(acv);
                        continue;
                    }
                    break;
                }
                if (S & 0x8000u) {  // unit complete
                    ++nb;
                    S &= 0x7Fu;
                    u = (cur >> 6) & 15u;
                    dc_slot = (cur >> 3) & 7u;
                    cur = __builtin_amdgcn_readlane(unit_word, u);
                    ac_slot = cur & 7u;
                    acv = ((ac_slot & 2u) ? e23 : e01) >> ((ac_slot & 1u) << 4);
                    acs = coop_step(acv);
                }
                if (S & 0x40u) break;
            }
            if (!more) break;
            S -= 64u;  // the same position, seen from the next window
            ws += 64u;
        }
        p = ws + (S & 0x7Fu);
        z = S >> 9;
    }
    p_io = p; u_io = u; z_io = z; nb_out = nb; dc_out = dc;
}

// ---- synchronisation, intra-sequence (paper, Algorithm 3, first loop) --------------------------------
// Workgroup w of an image covers the kWG subsequences base .. base+kWG-1, base = w*seq_len - overlap, and
// publishes the records of the last seq_len of them; the first `overlap` lanes only warm the chain up.

// STAGED: the workgroup's stretch of the stream is copied to LDS first (small subsequences); otherwise lanes
// read their words from global memory, one refill ahead, which leaves LDS to the tables and lets more
// workgroups share a CU (large subsequences).
// RST: the call has images with restart intervals.  Calls without get a kernel with none of that code in it (the
// intra-sequence kernel was measured 3 % slower on plain streams with it: registers and code layout).
// PHASE: kSyncAll = the whole of it in one kernel.  For calls with many more sequences than the chip holds at a time
// the work is split in two kernels.  kSyncHead is the same code up to the round in which at most P.handoff chains
// are still running; it leaves the records of all its lanes and the list of those chains in memory.  kSyncTail picks
// them up and runs the remaining rounds with the lanes reading the stream from memory (a handful of chains, each
// reading its words once).  The late rounds are chains of dependent symbols in a single wavefront or in one
// wavefront per chain, and what keeps the chip busy then is the number of sequences in flight: without the staged
// stream a workgroup needs a third of the LDS, and a CU holds eight of them instead of three.
constexpr int kSyncAll = 0, kSyncHead = 1, kSyncTail = 2;
constexpr uint32_t kHandMax = 128u;       // most chains a sequence may hand over
constexpr uint32_t kHandWords = 6u * kWG;  // per sequence: 4 x kWG record words, 3 x kHandMax chain words, the chain count
template <bool STAGED, bool RST, int PHASE>
__device__ __forceinline__ void sync_intra_body(const Params& P) {
    static_assert(PHASE != kSyncTail || !STAGED, "the second kernel reads the stream from memory");
    // Two symbols per step where the tables allow it (sync_symbol_pair); a workgroup whose stretch of the stream holds
    // the start of a restart interval takes the loop that knows their rules instead, one symbol per step.  Measured
    // on the 15360x8640 image: first kernel 0.85 -> 0.75 ms, second 1.00 -> 0.87 ms; 4096x4096 0.67 -> 0.59 ms; the
    // 256-image batch 0.40 -> 0.36 ms; nothing on images whose rounds are mostly walked by whole wavefronts
    // (1920x1088 with 128-bit subsequences).
    constexpr bool PAIRS = true;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    const uint32_t wg = blockIdx.x;
    const uint32_t ii = find_image(P, wg, [](const ImgDesc& d) { return d.seq0; });
    const ImgDesc D = image_desc(P, ii);
    const uint32_t nsub = P.st[ii].nsub;
    const int32_t base = (int32_t)((wg - D.seq0) * P.seq_len) - (int32_t)P.overlap;
    if (base >= (int32_t)nsub || (int32_t)((wg - D.seq0) * P.seq_len) >= (int32_t)nsub) return;  // nothing owned

    uint16_t* lut_s = reinterpret_cast<uint16_t*>(lds_raw);
    uint8_t* pair_s = reinterpret_cast<uint8_t*>(lut_s + P.lut_slots * (uint32_t)kLutEntries);
    uint32_t* sw = reinterpret_cast<uint32_t*>(pair_s + (PAIRS ? P.pair_slots * (uint32_t)kPairBytes : 0u));
    uint32_t* pnb = sw + kWG;
    uint32_t* pdc01 = pnb + kWG;
    uint32_t* pdc2 = pdc01 + kWG;
    // staging for packing the running chains: position; z (bits 0..7), u (8..11), target subsequence (12..).
    // The second kernel never has more than kHandMax chains.
    constexpr uint32_t kMv = PHASE == kSyncTail ? kHandMax : (uint32_t)kWG;
    uint32_t* mv_p = pdc2 + kWG;
    uint32_t* mv_s = mv_p + kMv;
    uint32_t* strm = mv_s + kMv;
    __shared__ uint32_t scratch[8];

    const uint32_t L = 1u << P.logL, wps = L >> 5;  // words per subsequence
    const uint32_t first = base < 0 ? 0u : (uint32_t)base;
    const uint32_t t0 = (uint32_t)((int32_t)first - base);                  // first lane with a subsequence
    const uint32_t t1 = min((uint32_t)kWG, (uint32_t)((int32_t)nsub - base));  // one past the last such lane
    const uint32_t first_word = first * wps;
    const uint32_t nwords = (t1 - t0) * wps + 4u;
    __shared__ UnitRow rows[8];
    __shared__ uint32_t pair_of_unit[8];
    stage_luts(P, D, lut_s);
    Syntax sx = stage_syntax(D, rows);
    if (PAIRS) {
        stage_pairs(P, D, pair_s, pair_of_unit);
        sx.pair_of_unit = pair_of_unit;
    }
    if (STAGED) stage_stream(P.stream + D.stream_off, first_word, nwords, strm);
    // scans with restart intervals: the bitmap of interval starts, for the bytes staged above
    uint32_t* bm_s = strm + (STAGED ? kWG * wps + 4u : 4u);
    const uint32_t bm_k0 = first_word >> 3;
    uint32_t seen = 0u;
    const bool bm_lds = (1u << P.logL) <= (uint32_t)kBitmapLdsMaxL;
    const uint32_t* bmap_img = P.bmap + D.bmap_off;
    if (RST && D.restart) seen = stage_bitmap(bmap_img, first_word, nwords, bm_s, bm_lds);
    auto bword = [&](uint32_t k) { return bm_lds ? bm_s[k - bm_k0] : bmap_img[k]; };
    bool restart = false;
    if (RST) restart = __syncthreads_or(seen != 0u) != 0;
    else __syncthreads();  // staged tables and stream are complete

    const uint32_t* gwords = reinterpret_cast<const uint32_t*>(P.stream + D.stream_off) + first_word;
    // cursor = word index inside the workgroup's window
    auto fetch = [&](uint32_t c) { return STAGED ? strm[c] : __builtin_bswap32(gwords[c]); };
    const uint32_t t = threadIdx.x;
    const bool valid = t >= t0 && t < t1;
    Lane l;
    BitWin w;
    int64_t dcacc = 0;
    uint32_t* handed = P.seq_rec + (size_t)wg * kHandWords;
    bool active = false;
    uint32_t tt = t + 1u;
    uint32_t waves_used = kWG / 64u;
    if (PHASE == kSyncTail) {
        // the records the first kernel left, and the chains that were still running
        if (valid) {
            sw[t] = handed[t];
            pnb[t] = handed[kWG + t];
            pdc01[t] = handed[2 * kWG + t];
            pdc2[t] = handed[3 * kWG + t];
        }
        const uint32_t n = handed[4u * kWG + 384u];
        active = t < n;
        if (active) {
            l.p = handed[4u * kWG + t];
            const uint32_t uz = handed[4u * kWG + 128u + t];
            l.u = uz >> 8;
            l.z = uz & 255u;
            l.nb = 0u;
            tt = handed[4u * kWG + 256u + t];
        }
        waves_used = (n + 63u) >> 6; if (waves_used == 0u) waves_used = 1u;
    } else if (valid) {
        const uint32_t i = (uint32_t)(base + (int32_t)t);
        l.p = i << P.logL; l.u = 0u; l.z = 0u; l.nb = 0u;
        win_init(w, l.p, (l.p >> 5) - first_word, fetch);
        prime(l, w, sx, lut_s);
        const uint32_t limit = (i + 1u) << P.logL;
        uint32_t crossed = 0u;
        if (restart) decode_span_sync_rst(l, w, limit, dcacc, crossed, sx, fetch, lut_s, bword);
        else if (PAIRS) decode_span_sync_pairs(l, w, limit, dcacc, sx, fetch, lut_s, pair_s);
        else decode_span_sync(l, w, limit, dcacc, sx, fetch, lut_s);
        sw[t] = pack_state(l.p - limit, l.z, l.u);
        pnb[t] = l.nb | (crossed << 31);
        pdc01[t] = pack_dc01(dcacc);
        pdc2[t] = pack_dc2(dcacc);
        active = t + 1u < t1;
    }
    // Overflow rounds: in round r the chain that started at subsequence c decodes subsequence c+r from its own
    // state and compares with the record left there one round earlier by the chain that started at c+1.
    // Chains drop out as they synchronise.  The chains still running are packed into the lowest lanes whenever
    // that frees a whole wavefront: a chain is (p, u, z, target), everything else is rebuilt from the staged
    // stream, so moving one costs two LDS words.  Between packings a round costs one barrier: the count of
    // running chains goes through one LDS word per wavefront, double-buffered by the parity of the round.
    // The wavefront-per-chain code does not know more than four tables.  In a workgroup that sees restart intervals
    // a chain may fall back to a single lane for a round (below): at most one chain per wavefront then, so that
    // such rounds never take longer than the packed ones they replace.
    const uint32_t coop_max = P.lut_slots > 4u ? 0u : (restart ? min(P.coop_max, P.sync_waves) : P.coop_max);
    uint32_t coop_n = 0u;
    bool first_tail_round = PHASE == kSyncTail;
    for (uint32_t round = 0u;; ++round) {
        const uint64_t bal = __ballot(active);
        uint32_t* cnt = scratch + ((round & 1u) << 2);
        if ((t & 63u) == 0u && t < (uint32_t)kWG) cnt[t >> 6] = (uint32_t)__popcll(bal);
        __syncthreads();  // also orders the records written in the previous round before their readers
        const uint32_t c0 = cnt[0], c1 = cnt[1], c2 = cnt[2], c3 = cnt[3];
        const uint32_t now = c0 + c1 + c2 + c3;
        if (PHASE == kSyncHead && now <= P.handoff) {  // the rest is the second kernel's
            const uint32_t wave = t >> 6;
            const uint32_t before = wave == 0u ? 0u : wave == 1u ? c0 : wave == 2u ? c0 + c1 : c0 + c1 + c2;
            const uint32_t rank = before + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
            if (active) {
                handed[4u * kWG + rank] = l.p;
                handed[4u * kWG + 128u + rank] = (l.u << 8) | l.z;
                handed[4u * kWG + 256u + rank] = tt;
            }
            if (t == 0u) handed[4u * kWG + 384u] = now;
            if (valid) {
                handed[t] = sw[t];
                handed[kWG + t] = pnb[t];
                handed[2 * kWG + t] = pdc01[t];
                handed[3 * kWG + t] = pdc2[t];
            }
            return;
        }
        if (now == 0u) break;
        if (now <= coop_max) {  // few chains left: hand them to whole wavefronts (below)
            const uint32_t wave = t >> 6;
            const uint32_t before = wave == 0u ? 0u : wave == 1u ? c0 : wave == 2u ? c0 + c1 : c0 + c1 + c2;
            const uint32_t rank = before + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
            if (active) {
                mv_p[rank] = l.p;
                mv_s[rank] = (tt << 12) | (l.u << 8) | l.z;
            }
            coop_n = now;
            __syncthreads();
            break;
        }
        if (((now + 63u) >> 6) < waves_used) {
            const uint32_t wave = t >> 6;
            const uint32_t before = wave == 0u ? 0u : wave == 1u ? c0 : wave == 2u ? c0 + c1 : c0 + c1 + c2;
            const uint32_t rank = before + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
            if (active) {
                mv_p[rank] = l.p;
                mv_s[rank] = (tt << 12) | (l.u << 8) | l.z;
            }
            __syncthreads();
            active = t < now;
            if (active) {
                l.p = mv_p[t];
                const uint32_t ms = mv_s[t];
                l.u = (ms >> 8) & 15u;
                l.z = ms & 255u;
                tt = ms >> 12;
                win_init(w, l.p, (l.p >> 5) - first_word, fetch);
                prime(l, w, sx, lut_s);
            }
            waves_used = (now + 63u) >> 6;
        }
        if (active) {
            l.nb = 0u;
            dcacc = 0;
            const uint32_t limit = ((uint32_t)(base + (int32_t)tt) + 1u) << P.logL;
            uint32_t crossed = 0u;
            if (PHASE == kSyncTail && first_tail_round) {
                win_init(w, l.p, (l.p >> 5) - first_word, fetch);
                prime(l, w, sx, lut_s);
            }
            if (restart) decode_span_sync_rst(l, w, limit, dcacc, crossed, sx, fetch, lut_s, bword);
            else if (PAIRS) decode_span_sync_pairs(l, w, limit, dcacc, sx, fetch, lut_s, pair_s);
            else decode_span_sync(l, w, limit, dcacc, sx, fetch, lut_s);
            const uint32_t x = pack_state(l.p - limit, l.z, l.u);
            const bool synced = x == sw[tt];
            sw[tt] = x;
            pnb[tt] = l.nb | (crossed << 31);
            pdc01[tt] = pack_dc01(dcacc);
            pdc2[tt] = pack_dc2(dcacc);
            ++tt;
            active = !synced && tt < t1;
        }
        first_tail_round = false;
    }
    // The same rounds with one chain per wavefront.  The chains keep their slot k < coop_n in a list held twice
    // (read from one copy, written to the other, swapped every round; mv_s = kCoopDone once a chain has
    // synchronised or reached the end of the sequence).  Every wavefront reads the whole list and takes the
    // running chains whose rank among them is its own number modulo the number of wavefronts (the four that hold
    // the lanes and the ones that are only here for this), so the work stays spread as chains drop out;
    // wavefront 0 carries the finished slots over.  One barrier per round.
    if (coop_n) {
        constexpr uint32_t kCoopDone = 0xFFFFFFFFu;
        // the compiler cannot know that these are the same in every lane (they come from the image descriptor and
        // the thread index); saying so keeps the chain's state in scalar registers
        const uint32_t wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63u;
        const uint32_t u_n = __builtin_amdgcn_readfirstlane(coop_n), u_t1 = __builtin_amdgcn_readfirstlane(t1);
        const uint32_t u_first = __builtin_amdgcn_readfirstlane(first_word), u_nwords = __builtin_amdgcn_readfirstlane(nwords);
        const uint32_t u_upm = __builtin_amdgcn_readfirstlane(sx.upm);
        const uint32_t u_waves = P.sync_waves;  // a power of two
        const int32_t u_base = (int32_t)__builtin_amdgcn_readfirstlane((uint32_t)base);
        const uint32_t unit_word = coop_unit_word(sx, lane);
        for (uint32_t par = 0u;; par ^= 1u) {
            const uint32_t rd = par << 6, wr = (par ^ 1u) << 6;
            const uint32_t mine = lane < u_n ? mv_s[rd + lane] : kCoopDone;
            const uint64_t running = __ballot(mine != kCoopDone);
            if (running == 0ull) break;
            if (wave == 0u && lane < u_n && mine == kCoopDone) mv_s[wr + lane] = kCoopDone;
            uint32_t rank = 0u;
            for (uint64_t m = running; m; m &= m - 1ull, ++rank) {
                if ((rank & (u_waves - 1u)) != wave) continue;
                const uint32_t k = (uint32_t)__ffsll((long long)m) - 1u;
                uint32_t cp = mv_p[rd + k];
                const uint32_t ms = __builtin_amdgcn_readfirstlane(mv_s[rd + k]);
                uint32_t cu = (ms >> 8) & 15u, cz = ms & 255u, cnb = 0u;
                const uint32_t ctt = ms >> 12;
                int64_t cdc = 0;
                const uint32_t limit = ((uint32_t)(u_base + (int32_t)ctt) + 1u) << P.logL;
                // The wavefront's decoder does not know the rules of restart intervals.  A chain whose stretch holds
                // no interval start does not need them (decode_span_sync_rst is the plain loop then); one whose
                // stretch does is decoded by a single lane for this round.
                uint32_t crossed = 0u;
                uint32_t B = kNoBoundary;
                if (restart) B = __builtin_amdgcn_readfirstlane(next_boundary(__builtin_amdgcn_readfirstlane(cp), limit + 64u, bword));
                if (B == kNoBoundary) {
                    coop_span_sync(cp, cu, cz, cnb, cdc, limit, u_first, u_nwords, unit_word, u_upm, P.lut_slots, fetch, lut_s);
                } else {
                    if (lane == 0u) {
                        Lane cl;
                        BitWin cw;
                        cl.p = cp; cl.u = cu; cl.z = cz; cl.nb = 0u;
                        win_init(cw, cl.p, (cl.p >> 5) - first_word, fetch);
                        prime(cl, cw, sx, lut_s);
                        decode_span_sync_rst(cl, cw, limit, cdc, crossed, sx, fetch, lut_s, bword);
                        cp = cl.p; cu = cl.u; cz = cl.z; cnb = cl.nb;
                    }
                    cp = __builtin_amdgcn_readfirstlane(cp);
                    cu = __builtin_amdgcn_readfirstlane(cu);
                    cz = __builtin_amdgcn_readfirstlane(cz);
                    cnb = __builtin_amdgcn_readfirstlane(cnb);
                    crossed = __builtin_amdgcn_readfirstlane(crossed);
                    const uint32_t dlo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)cdc);
                    const uint32_t dhi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)cdc >> 32));
                    cdc = (int64_t)(((uint64_t)dhi << 32) | (uint64_t)dlo);
                }
                const uint32_t x = pack_state(cp - limit, cz, cu);
                const bool synced = x == sw[ctt];
                if (lane == 0u) {
                    sw[ctt] = x;
                    pnb[ctt] = cnb | (crossed << 31);
                    pdc01[ctt] = pack_dc01(cdc);
                    pdc2[ctt] = pack_dc2(cdc);
                    mv_p[wr + k] = cp;
                    mv_s[wr + k] = (synced || ctt + 1u >= u_t1) ? kCoopDone : ((ctt + 1u) << 12) | (cu << 8) | cz;
                }
            }
            __syncthreads();
        }
    }
    if (valid && t >= P.overlap) {
        SInfo r;
        r.x = sw[t]; r.y = pnb[t]; r.z = pdc01[t]; r.w = pdc2[t];
        P.sinfo[D.sub0 + (uint32_t)(base + (int32_t)t)] = r;
    }
    // The published records continue the state the last warm-up lane ended in.  If the previous sequence ends
    // in that very state, the two sequences already form one chain and the inter-sequence kernel has nothing
    // to decode at this boundary.
    if (t == 0u) P.warm_x[wg] = (P.overlap > 0u && P.overlap - 1u >= t0) ? sw[P.overlap - 1u] : 0xFFFFFFFFu;
}

template <bool STAGED, bool RST>
__global__ __launch_bounds__(64 * kSyncWavesMax) void k_sync_intra(Params P) {
    sync_intra_body<STAGED, RST, kSyncAll>(P);
}
template <bool STAGED, bool RST>
__global__ __launch_bounds__(kWG) void k_sync_head(Params P) {
    sync_intra_body<STAGED, RST, kSyncHead>(P);
}
template <bool RST>
__global__ __launch_bounds__(kWG) void k_sync_tail(Params P) {
    sync_intra_body<false, RST, kSyncTail>(P);
}

// ---- synchronisation, inter-sequence (paper, Algorithm 3, second loop) ------------------------------
// One lane per sequence boundary: continue from the last record of sequence b into sequence b+1 until
// the state equals the recorded one or the sequence ends.  One wave64 per workgroup.

__global__ __launch_bounds__(64) void k_sync_inter(Params P) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    const uint32_t wg = blockIdx.x;
    const uint32_t ii = find_image(P, wg, [](const ImgDesc& d) { return d.bnd0; });
    const ImgDesc D = image_desc(P, ii);
    const uint32_t nsub = P.st[ii].nsub;
    const uint32_t b = (wg - D.bnd0) * 64u + threadIdx.x;
    const uint64_t gfirst = (uint64_t)(b + 1u) * P.seq_len;
    SInfo* rec = P.sinfo + D.sub0;
    uint32_t* warm = P.warm_x + D.seq0 + b + 1u;  // of the sequence that starts at this boundary
    // nothing to do where the sequence behind the boundary already continues the state the one before ends in
    uint32_t g = 0u, x0 = 0u;
    bool work = false;
    // The state words of records at a boundary are read here while the lane of the boundary before may be rewriting
    // them (and read again by the totals kernel, which opens another round if the two did not agree): single
    // 32-bit accesses, marked as such, with the rest of a record written before its state word.
    if (gfirst < nsub) {
        g = (uint32_t)gfirst;
        x0 = __atomic_load_n(&rec[g - 1u].x, __ATOMIC_RELAXED);
        work = *warm != x0;
    }
    if (!__syncthreads_or(work)) return;
    uint16_t* lut_s = reinterpret_cast<uint16_t*>(lds_raw);
    __shared__ UnitRow rows[8];
    stage_luts(P, D, lut_s);
    const Syntax sx = stage_syntax(D, rows);
    __syncthreads();
    const uint32_t* words = reinterpret_cast<const uint32_t*>(P.stream + D.stream_off);
    auto fetch = [&](uint32_t w) { return __builtin_bswap32(words[w]); };
    // Usually a handful of boundaries in a whole image have something to decode, and the kernel lasts as long as
    // the slowest of them.  With few in this workgroup, each is walked by the whole wavefront, one after the other
    // (same results as the lane's loop below; the wavefront's decoder does not know restart intervals).
    const uint64_t workers = __ballot(work);
    if (!D.restart && P.lut_slots <= 4u && __popcll(workers) <= kInterCoopMax) {
        const uint32_t lane = threadIdx.x;
        const uint32_t unit_word = coop_unit_word(sx, lane);
        const uint32_t u_upm = __builtin_amdgcn_readfirstlane(sx.upm);
        const uint32_t u_nsub = __builtin_amdgcn_readfirstlane(nsub);
        const uint32_t u_nwords = (u_nsub << (P.logL - 5u)) + 4u;
        for (uint64_t m = workers; m; m &= m - 1ull) {
            const uint32_t k = (uint32_t)__ffsll((long long)m) - 1u;
            uint32_t cg = __builtin_amdgcn_readlane(g, k);
            const uint32_t cx0 = __builtin_amdgcn_readlane(x0, k);
            const uint32_t cend = min(u_nsub, cg + P.seq_len);
            uint32_t cp = (cg << P.logL) + state_prel(cx0), cz = state_z(cx0), cu = state_u(cx0);
            bool first = true;
            for (;;) {
                uint32_t cnb = 0u;
                int64_t cdc = 0;
                const uint32_t limit = (cg + 1u) << P.logL;
                coop_span_sync(cp, cu, cz, cnb, cdc, limit, 0u, u_nwords, unit_word, u_upm, P.lut_slots, fetch, lut_s);
                const uint32_t x = pack_state(cp - limit, cz, cu);
                const bool synced = x == __atomic_load_n(&rec[cg].x, __ATOMIC_RELAXED);
                if (lane == 0u) {
                    if (first && !synced) atomicAdd(&P.status->inter_changed, 1u);
                    rec[cg].y = cnb;
                    rec[cg].z = pack_dc01(cdc);
                    rec[cg].w = pack_dc2(cdc);
                    __atomic_store_n(&rec[cg].x, x, __ATOMIC_RELAXED);
                }
                first = false;
                ++cg;
                if (synced || cg >= cend) break;
            }
        }
        if (work) *warm = x0;
        return;
    }
    if (!work) return;
    const uint32_t gend = min(nsub, g + P.seq_len);
    const uint32_t* bmap_img = P.bmap + D.bmap_off;
    auto bword = [&](uint32_t k) { return bmap_img[k]; };
    Lane l;
    BitWin w;
    l.p = (g << P.logL) + state_prel(x0);
    l.z = state_z(x0);
    l.u = state_u(x0);
    win_init(w, l.p, l.p >> 5, fetch);  // cursor = word index in the image's stream
    prime(l, w, sx, lut_s);
    bool first = true;
    for (;;) {
        l.nb = 0u;
        int64_t dcacc = 0;
        const uint32_t limit = (g + 1u) << P.logL;
        uint32_t crossed = 0u;
        if (D.restart) decode_span_sync_rst(l, w, limit, dcacc, crossed, sx, fetch, lut_s, bword);
        else decode_span_sync(l, w, limit, dcacc, sx, fetch, lut_s);
        SInfo r;
        r.x = pack_state(l.p - limit, l.z, l.u);
        r.y = l.nb | (crossed << 31);
        r.z = pack_dc01(dcacc);
        r.w = pack_dc2(dcacc);
        const bool synced = r.x == __atomic_load_n(&rec[g].x, __ATOMIC_RELAXED);
        if (first && !synced) atomicAdd(&P.status->inter_changed, 1u);
        first = false;
        rec[g].y = r.y;
        rec[g].z = r.z;
        rec[g].w = r.w;
        __atomic_store_n(&rec[g].x, r.x, __ATOMIC_RELAXED);
        ++g;
        if (synced || g >= gend) break;
    }
    *warm = x0;  // the sequence's records now continue this state
}

// ---- exclusive scan over s_info (paper, Algorithm 1: prefix sum on s_info.n) ---------------------------
// Level 1: totals of each group of kWG records.  Level 2: one workgroup per image scans the image's
// group totals.  Level 3 (inside the write kernel): scan within the group.

__global__ __launch_bounds__(kWG) void k_group_totals(Params P) {
    __shared__ uint32_t scratch[20];
    const uint32_t wg = blockIdx.x;
    const uint32_t ii = find_image(P, wg, [](const ImgDesc& d) { return d.grp0; });
    const ImgDesc D = image_desc_uniform(P, ii);
    const uint32_t nsub = P.st[ii].nsub;
    const uint32_t i = (wg - D.grp0) * kWG + threadIdx.x;
    SInfo r = {0u, 0u, 0u, 0u};
    if (i < nsub) r = P.sinfo[D.sub0 + i];
    Seg tot;
    wg_excl_segscan(seg_of_record(r), scratch, &tot);
    if (threadIdx.x == 0) P.grp_tot[wg] = seg_pack(tot);
    // The records of a sequence are those of a decoder that entered it in the state `warm_x` holds for it (the
    // state its workgroup's warm-up lanes arrived in, or the one an inter-sequence lane started from).  If the
    // sequence before it now ends in another state - an inter-sequence lane rewrote its last record in this very
    // round, after the lane of this boundary had looked - the states further on can still be right, and the write
    // pass will find nothing wrong, but the counts and DC sums of the sequence's first records belong to the other
    // entry state.  The boundaries inside this group are looked at here (at most four: a sequence has at least 65
    // subsequences), and the host runs another round if one is found.
    {
        const uint32_t i0 = (wg - D.grp0) * kWG;
        const uint32_t first = (i0 + P.seq_len - 1u) / P.seq_len;  // first sequence that starts in this group
        const uint32_t g = (first + threadIdx.x) * P.seq_len;
        if (threadIdx.x < 4u && g > 0u && g < nsub && g < i0 + (uint32_t)kWG) {
            const uint32_t seq = first + threadIdx.x;
            if (P.warm_x[D.seq0 + seq] != __atomic_load_n(&P.sinfo[D.sub0 + g - 1u].x, __ATOMIC_RELAXED)) atomicOr(&P.status->pending, 1u);
        }
    }
}

// one workgroup per image: exclusive prefix of the group totals
__global__ __launch_bounds__(kWG) void k_group_scan(Params P) {
    __shared__ uint32_t scratch[20];
    const uint32_t ii = blockIdx.x;
    const ImgDesc D = image_desc_uniform(P, ii);
    if (D.ngrp_max <= (uint32_t)kWG) return;  // images of up to 256 groups: the write kernel sums the totals itself
    const uint32_t ngrp = (P.st[ii].nsub + kWG - 1u) / kWG;
    // as in k_unstuff_scan: a run of consecutive groups per lane, one scan over the 256 joined runs
    const int4* tot = P.grp_tot + D.grp0;
    int4* pref = P.grp_pref + D.grp0;
    const uint32_t per = (ngrp + (uint32_t)kWG - 1u) / (uint32_t)kWG;
    const uint32_t k0 = min(threadIdx.x * per, ngrp), k1 = min(k0 + per, ngrp);
    Seg run = seg_zero();
    for (uint32_t k = k0; k < k1; ++k) run = seg_join(run, seg_unpack(tot[k]));
    Seg all;
    Seg ex = wg_excl_segscan(run, scratch, &all);
    for (uint32_t k = k0; k < k1; ++k) {
        pref[k] = seg_pack(ex);
        ex = seg_join(ex, seg_unpack(tot[k]));
    }
}

// ---- write pass (paper, Algorithm 1 last loop; Algorithm 2 with write = true) ---------------------------

template <bool STAGED>
__global__ __launch_bounds__(kWG) void k_write(Params P) {
    constexpr bool RST = true;  // (a variant without the restart code, as for k_sync_intra, was measured 2 % slower)
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    __shared__ uint32_t scratch[20];
    const uint32_t wg = blockIdx.x;
    const uint32_t ii = find_image(P, wg, [](const ImgDesc& d) { return d.grp0; });
    const ImgDesc D = image_desc_uniform(P, ii);
    const uint32_t nsub = P.st[ii].nsub;
    const uint32_t lg = wg - D.grp0;
    const uint32_t i0 = lg * kWG;
    if (i0 >= nsub) return;
    uint16_t* lut_s = reinterpret_cast<uint16_t*>(lds_raw);
    uint32_t* strm = reinterpret_cast<uint32_t*>(lut_s + P.lut_slots * (uint32_t)kLutEntries);

    const uint32_t L = 1u << P.logL, wps = L >> 5;
    const uint32_t nloc = min((uint32_t)kWG, nsub - i0);
    const uint32_t first_word = i0 * wps;
    const uint32_t nwords = nloc * wps + 4u;
    __shared__ UnitRow rows[8];
    // the lane's record, its predecessor's state and the totals of the groups before this one are asked for
    // first: their way from memory overlaps the staging below
    const uint32_t t = threadIdx.x;
    const uint32_t i = i0 + t;
    const bool valid = t < nloc;
    const SInfo* rec = P.sinfo + D.sub0;
    SInfo mine = {0u, 0u, 0u, 0u};
    uint32_t xprev = 0u;
    if (valid) {
        mine = rec[i];
        if (i > 0u) xprev = rec[i - 1u].x;
    }
    const bool few_groups = D.ngrp_max <= (uint32_t)kWG;
    int4 before = make_int4(0, 0, 0, 0);
    if (few_groups) {
        if (t < lg) before = P.grp_tot[D.grp0 + t];
    } else {
        before = P.grp_pref[wg];
    }
    stage_luts(P, D, lut_s);
    const Syntax sx = stage_syntax(D, rows);
    if (STAGED) stage_stream(P.stream + D.stream_off, first_word, nwords, strm);
    uint32_t* bm_s = strm + (STAGED ? kWG * wps + 4u : 4u);
    const uint32_t bm_k0 = first_word >> 3;
    uint32_t seen = 0u;
    const bool bm_lds = (1u << P.logL) <= (uint32_t)kBitmapLdsMaxL;
    const uint32_t* bmap_img = P.bmap + D.bmap_off;
    if (RST && D.restart) seen = stage_bitmap(bmap_img, first_word, nwords, bm_s, bm_lds);
    auto bword = [&](uint32_t k) { return bm_lds ? bm_s[k - bm_k0] : bmap_img[k]; };
    bool restart = false;  // interval starts in this group's stretch of the stream?
    if (RST) restart = __syncthreads_or(seen != 0u) != 0;
    else __syncthreads();

    // position of this lane's first data unit and its DC predictors: exclusive scan inside the group
    // plus the group's prefix
    Seg gp;
    if (few_groups) {
        wg_excl_segscan(seg_unpack(before), scratch, &gp);  // (all zero from lane lg on: the identity of the join)
    } else {
        gp = seg_unpack(before);
    }
    Seg grp_tot;
    const Seg ex = seg_join(gp, wg_excl_segscan(seg_of_record(mine), scratch, &grp_tot));
    const uint32_t grp_units = grp_tot.units;
    uint32_t unit = ex.units;
    int32_t pred0 = (int32_t)ex.d0, pred1 = (int32_t)ex.d1, pred2 = (int32_t)ex.d2;

    // The group clears the coefficients it is about to fill: those from where its first subsequence takes
    // over (data unit and zig-zag index) to where the next group's does; the last group goes on to the end of
    // the image.  The ranges of the groups tile the image, and a lane only stores inside its group's range.
    // Where the data units are dense (kDenseBitsPerUnit bits of stream or more per unit: most of their 64 slots hold a
    // value), the lanes lay down the few zeros of their own ranges as they go, chunk after chunk in address order,
    // and nothing is cleared up front: the clear would write every line a second time.  Where they are sparse, the
    // cooperative clear with full-width stores is far cheaper than one store per chunk and lane (measured: dense
    // treatment of the 1920x1088 4:4:4 image, 60 bits per unit, costs the kernel a third more time; on the noise half
    // of the 15360x8640 image, 340 bits per unit, it saves 8 %).  One decision per workgroup.
    const bool dense = ((uint64_t)nloc << P.logL) >= (uint64_t)kDenseBitsPerUnit * grp_units;
    if (!dense) {
        const uint64_t end_all = (uint64_t)D.total_units * 64u;
        const uint32_t x_in = i0 > 0u ? rec[i0 - 1u].x : 0u;
        const uint32_t x_out = rec[i0 + nloc - 1u].x;
        uint64_t a = (uint64_t)gp.units * 64u + state_z(x_in);
        uint64_t b = i0 + nloc >= nsub ? end_all : ((uint64_t)gp.units + grp_units) * 64u + state_z(x_out);
        if (i0 == 0u) a = 0u;
        if (b > end_all) b = end_all;
        if (a < b) {
            int16_t* c0 = P.coef + D.coef_off;
            uint64_t a8 = (a + 7u) & ~(uint64_t)7u;
            if (a8 > b) a8 = b;
            const uint64_t b8 = a8 + ((b - a8) & ~(uint64_t)7u);
            if (a + t < a8) c0[a + t] = 0;
            if (b8 + t < b) c0[b8 + t] = 0;
            uint4* body = reinterpret_cast<uint4*>(c0 + a8);
            const uint32_t n16 = (uint32_t)((b8 - a8) >> 3);
            const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
            for (uint32_t k = t; k < n16; k += kWG) body[k] = zero;
        }
    }
    __syncthreads();  // staged tables and stream are complete; the cleared range is in place
    if (!valid) return;

    const uint32_t* gwords = reinterpret_cast<const uint32_t*>(P.stream + D.stream_off) + first_word;
    auto fetch = [&](uint32_t c) { return STAGED ? strm[c] : __builtin_bswap32(gwords[c]); };
    int16_t* coef = P.coef + D.coef_off;
    // Coefficients leave the lane four at a time.  Every value as a store of its own makes 64 two-byte requests per
    // dense data unit, and the number of requests, not of bytes, is what the memory system charges for: the values
    // of four neighbouring slots (one aligned 8-byte chunk of the output) are gathered in a register pair and
    // stored together when the lane moves on to another chunk.  The zeros among them are the lane's own (the chunk
    // lies inside the range of slots this lane covers), except in the chunk the lane starts in, if it starts in
    // the middle of one, and in the chunk it ends in: those are shared with the neighbouring lanes and get their
    // values one by one.  (Eight slots per store were measured too: no faster on dense units, slower on sparse
    // ones.)
    const uint32_t S = unit * 64u + state_z(xprev);  // first slot of this lane's range
    const uint32_t S_chunk = S >> 2, S_low = S & 3u;
    uint64_t acc = 0ull;
    // chunk being gathered: 16 * data unit + (slot >> 2), from the chunk the lane's range starts in on (in a dense
    // workgroup zeros are laid down from the first slot on; in a sparse one a chunk left without a value costs a
    // store of zeros onto the cleared background, once per lane at most, and saves a test per chunk)
    uint32_t cur = S_chunk;
    const uint32_t shared_first = S_low != 0u ? S_chunk : 0xFFFFFFFFu;  // the first chunk, if a neighbour holds its start
    auto store8 = [&](uint32_t c, uint64_t a) { *reinterpret_cast<uint64_t*>(coef + (size_t)c * 4u) = a; };
    // elements lo .. hi-1 of chunk c, zeros included (chunks shared with a neighbouring lane, dense workgroups)
    auto put_part = [&](uint32_t c, uint64_t a, uint32_t lo, uint32_t hi) {
        int16_t* dst = coef + (size_t)c * 4u;
#pragma unroll
        for (uint32_t e = 0; e < 4u; ++e)
            if (e >= lo && e < hi) dst[e] = (int16_t)(uint16_t)(a >> (16u * e));
    };
    // the non-zero elements of chunk c (chunks shared with a neighbouring lane, onto the cleared background)
    auto put_nonzero = [&](uint32_t c, uint64_t a) {
        int16_t* dst = coef + (size_t)c * 4u;
#pragma unroll
        for (uint32_t e = 0; e < 4u; ++e) {
            const int16_t v = (int16_t)(uint16_t)(a >> (16u * e));
            if (v != 0) dst[e] = v;
        }
    };
    // the lane moves on to a later chunk: the one it leaves reaches up to its end inside the lane's range
    auto leave = [&]() {
        if (cur == shared_first) {
            if (dense) put_part(cur, acc, S_low, 4u);
            else put_nonzero(cur, acc);
        } else {
            store8(cur, acc);
        }
    };
    auto store = [&](uint32_t k, uint32_t at, int16_t v) {
        const uint32_t ck = k * 16u + (at >> 2);
        if (ck != cur) {
            leave();
            if (dense)
                for (uint32_t c = cur + 1u; c < ck; ++c) store8(c, 0ull);
            acc = 0ull;
            cur = ck;
        }
        acc |= (uint64_t)(uint16_t)v << ((at & 3u) * 16u);
    };
    Lane l;
    BitWin w;
    l.p = (i << P.logL) + state_prel(xprev);
    l.z = state_z(xprev);
    l.u = state_u(xprev);
    l.nb = 0u;
    pred0 = (int32_t)(int16_t)pred0; pred1 = (int32_t)(int16_t)pred1; pred2 = (int32_t)(int16_t)pred2;
    uint32_t flags = 0u;
    const uint32_t total = D.total_units;
    if (unit < total && unit % D.upm != l.u) flags |= kStUnit;
    const uint32_t limit = (i + 1u) << P.logL;
    if (unit < total) {
        win_init(w, l.p, (l.p >> 5) - first_word, fetch);
        prime(l, w, sx, lut_s);
        if (restart) decode_span_write_rst(l, w, limit, unit, total, D.restart * D.upm, pred0, pred1, pred2, sx, fetch, lut_s, store, flags, bword);
        else decode_span_write(l, w, limit, unit, total, pred0, pred1, pred2, sx, fetch, lut_s, store, flags);
    }
    if (dense) {
        // the rest of the lane's range, up to where the next lane takes over (or the image ends)
        const uint32_t E = unit < total ? unit * 64u + l.z : total * 64u;
        if (E > S) {
            const uint32_t E_chunk = E >> 2, E_low = E & 3u;
            const uint32_t lo = cur == S_chunk ? S_low : 0u, hi = cur == E_chunk ? E_low : 4u;
            if (lo == 0u && hi == 4u) store8(cur, acc);
            else put_part(cur, acc, lo, hi);
            for (uint32_t c = cur + 1u; c < E_chunk; ++c) store8(c, 0ull);
            if (E_low != 0u && E_chunk > cur) put_part(E_chunk, 0ull, 0u, E_low);
        }
    } else {
        put_nonzero(cur, acc);  // the last chunk may be shared with the next lane
    }
    // all restart markers must have been there (the first lane of the image speaks for it)
    if (RST && D.restart && i == 0u && P.st[ii].markers != D.nint - 1u) flags |= kStInvalid;
    // every lane checks the chain: unless the image is complete it must end in the recorded state
    if (unit < total) {
        if (l.p < limit || pack_state(l.p - limit, l.z, l.u) != mine.x) flags |= kStMismatch;
        if (i == nsub - 1u) flags |= kStShort;
    }
    if (flags) atomicOr(&P.status->flags, flags);
}

// ---- pixels: de-zigzag, dequantise, 8x8 IDCT, level shift, chroma replication, YCbCr -> RGB -------------
// (paper, Section 4.3; the colour steps are not in the paper).  A workgroup takes a run of consecutive
// MCUs of one MCU row, kPixBlocks data units at most, transforms them in LDS and writes the pixel
// rectangle they cover with row-contiguous stores.

constexpr int kBlkStride = 72;  // floats per data unit in LDS: 8 rows of 9 (one pad per row)
__device__ __constant__ uint8_t c_zigzag[64] = JPGD_ZIGZAG_LITERAL;

__global__ __launch_bounds__(kWG) void k_pixels(Params P) {
    __shared__ float blk[kPixBlocks * kBlkStride];
    __shared__ __attribute__((aligned(16))) float qf[3 * 64];
    const uint32_t wg = blockIdx.x;
    const uint32_t ii = find_image(P, wg, [](const ImgDesc& d) { return d.pix_wg0; });
    const ImgDesc D = image_desc_uniform(P, ii);
    const uint32_t lw = wg - D.pix_wg0;
    const uint32_t mrow = lw / D.pix_runs, run = lw % D.pix_runs;
    const uint32_t upm = D.upm;
    const uint32_t M = (uint32_t)kPixBlocks / upm;
    const uint32_t m0 = run * M;
    const uint32_t nm = min(M, D.mcus_x - m0);
    const uint32_t nblk = nm * upm;
    const uint32_t t = threadIdx.x;
    // The write kernel is complete when this kernel starts: its verdict goes to the waiting host from here, which
    // saves the dispatch of a kernel that would do nothing else.
    if (wg == 0u && t == 0u && P.verdict) {
        volatile uint32_t* host = P.verdict;
        host[0] = P.status->flags;
        host[1] = P.status->inter_changed;
        host[2] = P.status->pending;
        __threadfence_system();
        host[15] = P.ticket;
    }
    if (t < 3u * 64u) qf[t] = (float)P.qts[D.qt_off + t];
    // A lane always handles the same eighth of a data unit (256 is a multiple of 8): where its 8 coefficients
    // go inside the 8x9 tile is fixed, and is kept in registers.
    const uint32_t part = t & 7u;
    uint32_t zo[8];
#pragma unroll
    for (uint32_t e = 0; e < 8u; ++e) {
        const uint32_t rc = c_zigzag[part * 8u + e];
        zo[e] = (rc >> 3) * 9u + (rc & 7u);
    }
    __syncthreads();

    // load + dequantise + de-zigzag: 8 coefficients (16 bytes) per lane and step
    const int16_t* coef = P.coef + D.coef_off + (size_t)((size_t)mrow * D.mcus_x + m0) * upm * 64u;
    for (uint32_t j = t; j < nblk * 8u; j += kWG) {
        const uint32_t k = j >> 3;
        const uint32_t ku = upm == 1u ? 0u : (upm == 3u ? k % 3u : (upm == 4u ? (k & 3u) : k % 6u));
        const uint32_t comp = (D.sched_comp >> (ku * 4u)) & 15u;
        const uint4 raw = *reinterpret_cast<const uint4*>(coef + (size_t)j * 8u);
        const float4 qa = *reinterpret_cast<const float4*>(qf + comp * 64u + part * 8u);
        const float4 qb = *reinterpret_cast<const float4*>(qf + comp * 64u + part * 8u + 4u);
        float* tile = blk + k * kBlkStride;
        tile[zo[0]] = (float)(int16_t)(raw.x) * qa.x;
        tile[zo[1]] = (float)((int32_t)raw.x >> 16) * qa.y;
        tile[zo[2]] = (float)(int16_t)(raw.y) * qa.z;
        tile[zo[3]] = (float)((int32_t)raw.y >> 16) * qa.w;
        tile[zo[4]] = (float)(int16_t)(raw.z) * qb.x;
        tile[zo[5]] = (float)((int32_t)raw.z >> 16) * qb.y;
        tile[zo[6]] = (float)(int16_t)(raw.w) * qb.z;
        tile[zo[7]] = (float)((int32_t)raw.w >> 16) * qb.w;
    }
    __syncthreads();
    // columns, then rows
    for (uint32_t j = t; j < nblk * 8u; j += kWG) {
        float* b = blk + (j >> 3) * kBlkStride + (j & 7u);
        float v0 = b[0], v1 = b[9], v2 = b[18], v3 = b[27], v4 = b[36], v5 = b[45], v6 = b[54], v7 = b[63];
        idct8(v0, v1, v2, v3, v4, v5, v6, v7);
        b[0] = v0; b[9] = v1; b[18] = v2; b[27] = v3; b[36] = v4; b[45] = v5; b[54] = v6; b[63] = v7;
    }
    __syncthreads();
    for (uint32_t j = t; j < nblk * 8u; j += kWG) {
        float* b = blk + (j >> 3) * kBlkStride + (j & 7u) * 9u;
        float v0 = b[0], v1 = b[1], v2 = b[2], v3 = b[3], v4 = b[4], v5 = b[5], v6 = b[6], v7 = b[7];
        v0 += kLevelShiftDc;  // the level shift of +128 on all eight outputs, as one addition to the row's DC term
        idct8(v0, v1, v2, v3, v4, v5, v6, v7);
        b[0] = v0; b[1] = v1; b[2] = v2; b[3] = v3; b[4] = v4; b[5] = v5; b[6] = v6; b[7] = v7;
    }
    __syncthreads();

    // output
    // (sampling factors are 1 or 2: shifts instead of divisions; the one division by a free number, the
    // groups per row, goes through a reciprocal that is exact for the few hundred items of a workgroup)
    const uint32_t hs = D.hs, vs = D.vs, ncomp = D.ncomp;
    const uint32_t lhs = hs >> 1, lvs = vs >> 1;          // log2 of 1 or 2
    const uint32_t mcu_w = 8u * hs, mcu_h = 8u * vs, lmw = 3u + lhs;
    const uint32_t region_w = nm * mcu_w;
    const uint32_t groups_per_row = region_w >> 2;
    const float inv_gpr = 1.0f / (float)groups_per_row;
    uint8_t* pix = P.pixels + D.pix_off;
    const uint32_t x_base = m0 * mcu_w, y_base = mrow * mcu_h;
    if (P.planar) {
        // The paper's own output (Section 3: one array per colour channel): every component at its own
        // resolution, rounded and clamped.  Luma plane first, then Cb, then Cr.
        auto put4 = [&](uint8_t* dst, const float* src, uint32_t left, bool word_ok) {
            uint32_t w = pack_u8(src[0], 0u, 0u);
            w = pack_u8(src[1], 1u, w); w = pack_u8(src[2], 2u, w); w = pack_u8(src[3], 3u, w);
            if (left >= 4u && word_ok) {
                *reinterpret_cast<uint32_t*>(dst) = w;
            } else {
                dst[0] = (uint8_t)w;
                if (left > 1u) dst[1] = (uint8_t)(w >> 8);
                if (left > 2u) dst[2] = (uint8_t)(w >> 16);
                if (left > 3u) dst[3] = (uint8_t)(w >> 24);
            }
        };
        const bool y_words = (D.width & 3u) == 0u && (reinterpret_cast<size_t>(pix) & 3u) == 0u;
        for (uint32_t j = t; j < groups_per_row * mcu_h; j += kWG) {
            const uint32_t py = (uint32_t)(((float)j + 0.5f) * inv_gpr), px0 = (j - py * groups_per_row) * 4u;
            const uint32_t gy = y_base + py, gx0 = x_base + px0;
            if (gy >= D.height || gx0 >= D.width) continue;
            const uint32_t m = px0 >> lmw, xin = px0 & (mcu_w - 1u);
            const float* yb = blk + (m * upm + (py >> 3) * hs + (xin >> 3)) * kBlkStride + (py & 7u) * 9u + (xin & 7u);
            put4(pix + (size_t)gy * D.width + gx0, yb, D.width - gx0, y_words);
        }
        if (ncomp == 3u) {
            const uint32_t cw = (D.width + hs - 1u) >> lhs, ch = (D.height + vs - 1u) >> lvs;  // chroma plane size
            uint8_t* cplane = pix + (size_t)D.width * D.height;
            const bool c_words = (cw & 3u) == 0u && (reinterpret_cast<size_t>(cplane) & 3u) == 0u && (((size_t)cw * ch) & 3u) == 0u;
            const uint32_t gpr_c = nm * 2u;  // groups of 4 samples per chroma row of this workgroup
            for (uint32_t j = t; j < gpr_c * 16u; j += kWG) {
                const uint32_t c = j >= gpr_c * 8u ? 1u : 0u;
                const uint32_t r = j - c * gpr_c * 8u;
                const uint32_t py = (uint32_t)(((float)r + 0.5f) / (float)gpr_c), g = r - py * gpr_c;
                const uint32_t m = g >> 1, xin = (g & 1u) * 4u;
                const uint32_t gy = mrow * 8u + py, gx0 = (m0 + m) * 8u + xin;
                if (gy >= ch || gx0 >= cw) continue;
                const float* cb = blk + (m * upm + hs * vs + c) * kBlkStride + py * 9u + xin;
                put4(cplane + (size_t)c * cw * ch + (size_t)gy * cw + gx0, cb, cw - gx0, c_words);
            }
        }
        return;
    }
    // RGB or gray: a lane produces the 8 (gray) or 24 bytes of eight horizontally adjacent pixels -- one row of a
    // luma data unit -- as whole words.  The colour terms of a chroma sample are computed once (a sample serves two
    // of the pixels when chroma is subsampled horizontally); each output sample then costs one addition and one
    // conversion that also puts the byte in its place.
    // (all factors below are far under 2^24: the 24-bit multiply runs at full rate, the 32-bit one at a quarter)
    const bool aligned = (((size_t)D.width * ncomp) & 3u) == 0u && ((reinterpret_cast<size_t>(pix)) & 3u) == 0u;
    const uint32_t row_bytes = D.width * ncomp;  // a frame header holds the width in 16 bits
    const uint32_t rows8 = region_w >> 3;         // groups of 8 pixels per row of the workgroup's rectangle
    const float inv_rows8 = 1.0f / (float)rows8;
    // bytes in memory: R0 G0 B0 R1 | G1 B1 R2 G2 | B2 R3 G3 B3
    auto pack12 = [](uint32_t& wa, uint32_t& wb, uint32_t& wc, float y0, float y1, float y2, float y3,
                     const ChromaTerms& c0, const ChromaTerms& c1, const ChromaTerms& c2, const ChromaTerms& c3) {
        wa = pack_u8(y0 + c0.r, 0u, wa); wa = pack_u8(y0 + c0.g, 1u, wa); wa = pack_u8(y0 + c0.b, 2u, wa);
        wa = pack_u8(y1 + c1.r, 3u, wa); wb = pack_u8(y1 + c1.g, 0u, wb); wb = pack_u8(y1 + c1.b, 1u, wb);
        wb = pack_u8(y2 + c2.r, 2u, wb); wb = pack_u8(y2 + c2.g, 3u, wb); wc = pack_u8(y2 + c2.b, 0u, wc);
        wc = pack_u8(y3 + c3.r, 1u, wc); wc = pack_u8(y3 + c3.g, 2u, wc); wc = pack_u8(y3 + c3.b, 3u, wc);
    };
    for (uint32_t j = t; j < rows8 * mcu_h; j += kWG) {
        const uint32_t py = (uint32_t)(((float)j + 0.5f) * inv_rows8), px0 = (j - __umul24(py, rows8)) * 8u;
        const uint32_t gy = y_base + py, gx0 = x_base + px0;
        if (gy >= D.height || gx0 >= D.width) continue;
        const uint32_t m = px0 >> lmw, xin = px0 & (mcu_w - 1u);  // xin: 0, or 8 in the right half of a 16-wide MCU
        const uint32_t mu = __umul24(m, upm);
        const float* yb = blk + __umul24(mu + __umul24(py >> 3, hs) + (xin >> 3), (uint32_t)kBlkStride) + (py & 7u) * 9u;
        const float y0 = yb[0], y1 = yb[1], y2 = yb[2], y3 = yb[3], y4 = yb[4], y5 = yb[5], y6 = yb[6], y7 = yb[7];
        uint32_t w0 = 0u, w1 = 0u, w2 = 0u, w3 = 0u, w4 = 0u, w5 = 0u;
        if (ncomp == 1u) {
            w0 = pack_u8(y0, 0u, w0); w0 = pack_u8(y1, 1u, w0); w0 = pack_u8(y2, 2u, w0); w0 = pack_u8(y3, 3u, w0);
            w1 = pack_u8(y4, 0u, w1); w1 = pack_u8(y5, 1u, w1); w1 = pack_u8(y6, 2u, w1); w1 = pack_u8(y7, 3u, w1);
        } else {
            const float* cbb = blk + __umul24(mu + hs * vs, (uint32_t)kBlkStride) + (py >> lvs) * 9u + (xin >> lhs);
            const float* crb = cbb + kBlkStride;
            if (hs == 2u) {  // (the two cases are written out so that neither pays register moves for the other)
                const ChromaTerms a = chroma_terms(cbb[0], crb[0]), b = chroma_terms(cbb[1], crb[1]);
                pack12(w0, w1, w2, y0, y1, y2, y3, a, a, b, b);
                const ChromaTerms c = chroma_terms(cbb[2], crb[2]), d = chroma_terms(cbb[3], crb[3]);
                pack12(w3, w4, w5, y4, y5, y6, y7, c, c, d, d);
            } else {
                {
                    const ChromaTerms a = chroma_terms(cbb[0], crb[0]), b = chroma_terms(cbb[1], crb[1]);
                    const ChromaTerms c = chroma_terms(cbb[2], crb[2]), d = chroma_terms(cbb[3], crb[3]);
                    pack12(w0, w1, w2, y0, y1, y2, y3, a, b, c, d);
                }
                {
                    const ChromaTerms a = chroma_terms(cbb[4], crb[4]), b = chroma_terms(cbb[5], crb[5]);
                    const ChromaTerms c = chroma_terms(cbb[6], crb[6]), d = chroma_terms(cbb[7], crb[7]);
                    pack12(w3, w4, w5, y4, y5, y6, y7, a, b, c, d);
                }
            }
        }
        uint8_t* dst = pix + (size_t)gy * row_bytes + __umul24(gx0, ncomp);
        if (gx0 + 8u <= D.width && aligned) {
            uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
            d32[0] = w0;
            d32[1] = w1;
            if (ncomp == 3u) {
                d32[2] = w2; d32[3] = w3; d32[4] = w4; d32[5] = w5;
            }
        } else {
            const uint32_t nbytes = min(8u, D.width - gx0) * ncomp;
            for (uint32_t e = 0; e < nbytes; ++e) {
                const uint32_t w = e < 4u ? w0 : (e < 8u ? w1 : (e < 12u ? w2 : (e < 16u ? w3 : (e < 20u ? w4 : w5))));
                dst[e] = (uint8_t)(w >> (8u * (e & 3u)));
            }
        }
    }
}

// ---- pixels at reduced size ------------------------------------------------------------------------------
// Output at 1/2, 1/4 or 1/8 of the size straight from the coefficients: of every data unit only the N x N lowest
// frequencies are read, N = 4, 2, 1, and the N-point inverse transform is applied to them,
//   f(y,x) = 1/4 sum_{u<N} sum_{v<N} C(u) C(v) F(v,u) cos((2x+1) u pi/(2N)) cos((2y+1) v pi/(2N)),
// with the 8-point transform's factor, so that a unit holding only a DC term keeps its value.  Everything after
// that is as at full size: level shift, chroma replicated by the sampling factors, colour matrix, one rounding,
// crop to ceil(width / d) x ceil(height / d).  (The paper's decoder ends with the full-size transform, Section 4.3,
// and names it as the stage that now limits the decoder; this path reads the same coefficients and skips most of it.)

// c_basis*[x * N + u] = 1/2 C(u) cos((2x+1) u pi / (2N))
#define JPGD_BASIS4_LITERAL                                                                            \
    {0.35355339059327379f, 0.46193976625564337f, 0.35355339059327379f, 0.19134171618254489f,            \
     0.35355339059327379f, 0.19134171618254489f, -0.35355339059327379f, -0.46193976625564337f,          \
     0.35355339059327379f, -0.19134171618254489f, -0.35355339059327379f, 0.46193976625564337f,          \
     0.35355339059327379f, -0.46193976625564337f, 0.35355339059327379f, -0.19134171618254489f}
#define JPGD_BASIS2_LITERAL {0.35355339059327379f, 0.35355339059327379f, 0.35355339059327379f, -0.35355339059327379f}
// (the same values twice: as compile-time constants for sums whose position is unrolled, and in constant memory for
// the table a lane indexes with its row)
constexpr float c_basis4_host[16] = JPGD_BASIS4_LITERAL;
constexpr float c_basis2_host[4] = JPGD_BASIS2_LITERAL;
__device__ __constant__ float c_basis4[16] = {
    0.35355339059327379f, 0.46193976625564337f, 0.35355339059327379f, 0.19134171618254489f,
    0.35355339059327379f, 0.19134171618254489f, -0.35355339059327379f, -0.46193976625564337f,
    0.35355339059327379f, -0.19134171618254489f, -0.35355339059327379f, 0.46193976625564337f,
    0.35355339059327379f, -0.46193976625564337f, 0.35355339059327379f, -0.19134171618254489f};
__device__ __constant__ float c_basis2[4] = {0.35355339059327379f, 0.35355339059327379f,
                                             0.35355339059327379f, -0.35355339059327379f};

// natural (row-major) position -> zig-zag position: the inverse of the zig-zag literal, made at compile time
struct UnZigzag {
    uint8_t at[64];
    constexpr UnZigzag() : at{} {
        constexpr uint8_t zz[64] = JPGD_ZIGZAG_LITERAL;
        for (int i = 0; i < 64; ++i) at[zz[i]] = (uint8_t)i;
    }
};
__device__ __constant__ UnZigzag c_unzigzag = UnZigzag();

template <int N>
__global__ __launch_bounds__(kWG) void k_pixels_scaled(Params P) {
    constexpr uint32_t NN = N * N;
    constexpr uint32_t lN = N == 4 ? 2u : (N == 2 ? 1u : 0u);   // log2 N
    __shared__ float fin[kPixBlocksScaled * NN];   // dequantised low frequencies, [unit][v * N + u]
    __shared__ float smp[kPixBlocksScaled * NN];   // samples, level shift applied, [unit][y * N + x]
    __shared__ float bs[NN];
    const uint32_t wg = blockIdx.x;
    const uint32_t ii = find_image(P, wg, [](const ImgDesc& d) { return d.pix_wg0; });
    const ImgDesc D = image_desc_uniform(P, ii);
    const uint32_t lw = wg - D.pix_wg0;
    const uint32_t mrow = lw / D.pix_runs, run = lw % D.pix_runs;
    const uint32_t upm = D.upm;
    const uint32_t M = (uint32_t)kPixBlocksScaled / upm;
    const uint32_t m0 = run * M;
    const uint32_t nm = min(M, D.mcus_x - m0);
    const uint32_t nblk = nm * upm;
    const uint32_t t = threadIdx.x;
    if (wg == 0u && t == 0u && P.verdict) {  // the verdict of the write kernel, as in k_pixels
        volatile uint32_t* host = P.verdict;
        host[0] = P.status->flags;
        host[1] = P.status->inter_changed;
        host[2] = P.status->pending;
        __threadfence_system();
        host[15] = P.ticket;
    }
    if (t < NN) bs[t] = N == 4 ? c_basis4[t] : (N == 2 ? c_basis2[t & 3u] : 0.35355339059327379f);
    // A lane always fetches the same frequency (256 is a multiple of N * N): its zig-zag position is looked up once.
    const uint32_t e = t & (NN - 1u);
    const uint32_t zpos = c_unzigzag.at[(e >> lN) * 8u + (e & (N - 1u))];
    const int16_t* coef = P.coef + D.coef_off + (size_t)((size_t)mrow * D.mcus_x + m0) * upm * 64u;
    const uint16_t* qt = P.qts + D.qt_off + zpos;
    const float q0 = (float)qt[0], q1 = (float)qt[64], q2 = (float)qt[128];
    for (uint32_t j = t; j < nblk * NN; j += kWG) {
        const uint32_t k = j >> (2u * lN);
        const uint32_t ku = upm == 1u ? 0u : (upm == 3u ? k % 3u : (upm == 4u ? (k & 3u) : k % 6u));
        const uint32_t comp = (D.sched_comp >> (ku * 4u)) & 15u;
        fin[j] = (float)coef[(size_t)k * 64u + zpos] * (comp == 0u ? q0 : (comp == 1u ? q1 : q2));
    }
    __syncthreads();
    // one lane per row of a unit's N x N samples: first the sum over the vertical frequencies for its row (weights
    // from the basis table in LDS, they depend on the row), then the N outputs (weights are constants)
    for (uint32_t j = t; j < nblk * N; j += kWG) {
        const uint32_t k = j >> lN, y = j & (N - 1u);
        const float* F = fin + k * NN;
        float g[N];
#pragma unroll
        for (uint32_t u = 0; u < (uint32_t)N; ++u) g[u] = 0.0f;
#pragma unroll
        for (uint32_t v = 0; v < (uint32_t)N; ++v) {
            const float w = bs[y * N + v];
#pragma unroll
            for (uint32_t u = 0; u < (uint32_t)N; ++u) g[u] = __builtin_fmaf(w, F[v * N + u], g[u]);
        }
#pragma unroll
        for (uint32_t x = 0; x < (uint32_t)N; ++x) {
            float acc = 128.0f;
#pragma unroll
            for (uint32_t u = 0; u < (uint32_t)N; ++u)
                acc = __builtin_fmaf(N == 4 ? c_basis4_host[x * 4u + u] : (N == 2 ? c_basis2_host[(x * 2u + u) & 3u] : 0.35355339059327379f), g[u], acc);
            smp[k * NN + y * N + x] = acc;
        }
    }
    __syncthreads();

    const uint32_t hs = D.hs, vs = D.vs, ncomp = D.ncomp;
    const uint32_t lhs = hs >> 1, lvs = vs >> 1;
    const uint32_t ls = 3u - lN;                                  // log2 of the scale denominator
    const uint32_t ow = (D.width + (1u << ls) - 1u) >> ls, oh = (D.height + (1u << ls) - 1u) >> ls;
    uint8_t* pix = P.pixels + D.pix_off;
    // sample (py, px) of the rectangle that component units [u0, u0 + ux * uy) of the workgroup's MCUs cover
    // (ux x uy units of N x N samples per MCU)
    auto sample = [&](uint32_t u0, uint32_t lux, uint32_t py, uint32_t px) {
        const uint32_t lmw = lN + lux;                            // log2 of the samples per MCU row
        const uint32_t m = px >> lmw, xin = px & ((1u << lmw) - 1u);
        const uint32_t unit = m * upm + u0 + ((py >> lN) << lux) + (xin >> lN);
        return smp[unit * NN + ((py & (N - 1u)) << lN) + (xin & (N - 1u))];
    };
    auto put = [&](uint8_t* dst, const uint32_t* w, uint32_t nbytes, bool words) {
        if (words) {
            for (uint32_t e = 0; e < nbytes / 4u; ++e) reinterpret_cast<uint32_t*>(dst)[e] = w[e];
        } else {
            for (uint32_t e = 0; e < nbytes; ++e) dst[e] = (uint8_t)(w[e >> 2] >> (8u * (e & 3u)));
        }
    };
    if (P.planar) {
        // component planes at reduced size, one after the other: plane c has ceil(plane_w / d) x ceil(plane_h / d) samples
        size_t plane_off = 0;
        for (uint32_t c = 0; c < ncomp; ++c) {
            const uint32_t lux = c == 0u ? lhs : 0u, luy = c == 0u ? lvs : 0u;
            const uint32_t u0 = c == 0u ? 0u : hs * vs + c - 1u;
            const uint32_t full_w = c == 0u ? D.width : (D.width + hs - 1u) >> lhs;
            const uint32_t full_h = c == 0u ? D.height : (D.height + vs - 1u) >> lvs;
            const uint32_t pw = (full_w + (1u << ls) - 1u) >> ls, ph = (full_h + (1u << ls) - 1u) >> ls;
            uint8_t* plane = pix + plane_off;
            plane_off += (size_t)pw * ph;
            const uint32_t region_w = nm << (lN + lux), region_h = 1u << (lN + luy);
            const uint32_t gpr = (region_w + 3u) >> 2;
            const uint32_t x_base = m0 << (lN + lux), y_base = mrow << (lN + luy);
            const bool words_ok = (pw & 3u) == 0u && (reinterpret_cast<size_t>(plane) & 3u) == 0u;
            for (uint32_t j = t; j < gpr * region_h; j += kWG) {
                const uint32_t py = j / gpr, px0 = (j - py * gpr) * 4u;
                const uint32_t gy = y_base + py, gx0 = x_base + px0;
                if (gy >= ph || gx0 >= pw) continue;
                const uint32_t cnt = min(4u, min(region_w - px0, pw - gx0));
                uint32_t w[1] = {0u};
                w[0] = pack_u8(sample(u0, lux, py, px0), 0u, w[0]);
                w[0] = pack_u8(sample(u0, lux, py, min(px0 + 1u, region_w - 1u)), 1u, w[0]);
                w[0] = pack_u8(sample(u0, lux, py, min(px0 + 2u, region_w - 1u)), 2u, w[0]);
                w[0] = pack_u8(sample(u0, lux, py, min(px0 + 3u, region_w - 1u)), 3u, w[0]);
                put(plane + (size_t)gy * pw + gx0, w, cnt, cnt == 4u && words_ok);
            }
        }
        return;
    }
    // gray or RGB: a lane produces four horizontally adjacent pixels
    const uint32_t region_w = nm << (lN + lhs), region_h = 1u << (lN + lvs);
    const uint32_t gpr = (region_w + 3u) >> 2;
    const uint32_t x_base = m0 << (lN + lhs), y_base = mrow << (lN + lvs);
    const uint32_t row_bytes = ow * ncomp;
    const bool words_ok = (row_bytes & 3u) == 0u && (reinterpret_cast<size_t>(pix) & 3u) == 0u;
    for (uint32_t j = t; j < gpr * region_h; j += kWG) {
        const uint32_t py = j / gpr, px0 = (j - py * gpr) * 4u;
        const uint32_t gy = y_base + py, gx0 = x_base + px0;
        if (gy >= oh || gx0 >= ow) continue;
        const uint32_t cnt = min(4u, min(region_w - px0, ow - gx0));
        uint32_t w[3] = {0u, 0u, 0u};
        float yv[4];
        ChromaTerms ct[4];
#pragma unroll
        for (uint32_t e = 0; e < 4u; ++e) {
            const uint32_t px = min(px0 + e, region_w - 1u);
            yv[e] = sample(0u, lhs, py, px);
            if (ncomp == 3u) {
                const float cb = sample(hs * vs, 0u, py >> lvs, px >> lhs), cr = sample(hs * vs + 1u, 0u, py >> lvs, px >> lhs);
                ct[e] = chroma_terms(cb, cr);
            }
        }
        if (ncomp == 1u) {
            w[0] = pack_u8(yv[0], 0u, w[0]); w[0] = pack_u8(yv[1], 1u, w[0]);
            w[0] = pack_u8(yv[2], 2u, w[0]); w[0] = pack_u8(yv[3], 3u, w[0]);
        } else {
            // bytes in memory: R0 G0 B0 R1 | G1 B1 R2 G2 | B2 R3 G3 B3
            w[0] = pack_u8(yv[0] + ct[0].r, 0u, w[0]); w[0] = pack_u8(yv[0] + ct[0].g, 1u, w[0]); w[0] = pack_u8(yv[0] + ct[0].b, 2u, w[0]);
            w[0] = pack_u8(yv[1] + ct[1].r, 3u, w[0]); w[1] = pack_u8(yv[1] + ct[1].g, 0u, w[1]); w[1] = pack_u8(yv[1] + ct[1].b, 1u, w[1]);
            w[1] = pack_u8(yv[2] + ct[2].r, 2u, w[1]); w[1] = pack_u8(yv[2] + ct[2].g, 3u, w[1]); w[2] = pack_u8(yv[2] + ct[2].b, 0u, w[2]);
            w[2] = pack_u8(yv[3] + ct[3].r, 1u, w[2]); w[2] = pack_u8(yv[3] + ct[3].g, 2u, w[2]); w[2] = pack_u8(yv[3] + ct[3].b, 3u, w[2]);
        }
        put(pix + (size_t)gy * row_bytes + (size_t)gx0 * ncomp, w, cnt * ncomp, cnt == 4u && words_ok);
    }
}

}  // namespace jpgd
