// Internal definitions shared by the host code and the gfx950 kernels.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define JPGD_HD __host__ __device__ __forceinline__
#else
#define JPGD_HD inline
#endif

namespace jpgd {

// ---- geometry of the parallel decomposition (paper, Section 4.1, Algorithm 1) ----------------
// subsequence : L bits of the unstuffed stream, one lane
// sequence    : the subsequences one workgroup synchronises among itself ("b" in the paper)
constexpr int kWG = 256;          // lanes per workgroup of the sync and write kernels
// Streams with restart intervals: the synchronisation and write kernels keep the interval-start bitmap of their
// stretch of the stream in LDS up to this subsequence size.  Beyond it the copy (4 KB at 1024 bits) would cost a
// third of the workgroups a CU can hold, and a lane asks for a bitmap word only once or twice per subsequence,
// so the words are read from memory instead.
constexpr int kBitmapLdsMaxL = 256;
constexpr int kMaxOverlap = 191;  // warm-up lanes a sequence may borrow from its predecessor

// ---- Huffman lookup tables ---------------------------------------------------------------------
// One table = kLutL1 first-level entries indexed by the next kLutK bits, followed by up to kLutL2
// second-level entries for codewords longer than kLutK bits.  uint16 entries:
//   bits 0..4   bits the symbol takes: codeword (1..16) plus value bits, at most 31
//   bits 5..8   number of value bits that follow the codeword, 0..15
//   bits 9..14  zig-zag slots the symbol covers: run+1 for a coefficient, 1 for a DC symbol, 16 for
//               ZRL, 63 for end-of-block (any z >= 1 plus 63 reaches 64 = unit complete), and 0 for
//               "no codeword starts with these bits" (one bit taken: skip it, state unchanged)
//   bit 15      0
//   first-level escape: bit 15 = 1, bits 0..2 = number of further bits that index the second level,
//               bits 3..10 = half the offset of the subtable inside the second level
// Bound on the second level: codes of one length are consecutive, so those of length l > kLutK touch
// at most n_l / 2^(l-kLutK) + 2 first-level prefixes; summed over l = 11..16 with at most 256 symbols
// this is below 510 entries; two more hold the shared "no codeword" record.
constexpr int kLutK = 10;
constexpr int kLutL1 = 1 << kLutK;
constexpr int kLutL2 = 512;
constexpr int kLutEntries = kLutL1 + kLutL2;
constexpr int kMaxSlots = 6;  // up to 3 DC and 3 AC tables per image (one pair per component)
constexpr uint32_t kAdvEob = 63u;
// Per AC table, one byte per first-level index: the symbol behind the one the entry describes, where the index
// holds it (build_pairs; used by the synchronisation pass).  In memory the pair bytes of an image's tables follow
// its kMaxSlots table slots: a set of tables takes kLutSetEntries uint16.
constexpr int kPairBytes = kLutL1;
constexpr int kMaxPairs = kMaxSlots / 2;
constexpr int kLutSetEntries = kMaxSlots * kLutEntries + kMaxPairs * kPairBytes / 2;

// Intra-sequence synchronisation: with at most one and a half chains per wavefront of the workgroup still running,
// each chain is decoded by a whole wavefront.  Measured on 1920x1088 4:4:4 (128-bit subsequences) and on 4096x4096
// and 15360x8640 4:2:0 (1024 bits): with four wavefronts 4 to 8 chains are within noise of each other and 16 is
// slower than never doing it on the large images; with eight wavefronts 12 is best, with sixteen 24.
constexpr uint32_t kCoopMax = 6u;  // for the kWG / 64 wavefronts that hold the lanes
// The workgroup may have more wavefronts than those: the others do nothing but take chains in these rounds, so
// that fewer chains share a wavefront (a CU has 32 wavefront slots and a sequence's tail leaves most of them idle).
constexpr int kSyncWavesMax = 16;
// Intra-sequence synchronisation as two kernels: calls with at least this many sequences (twice what the chip holds
// at a time with 1024-bit subsequences), and the number of running chains at which a sequence changes kernel
// (48 and 64 are within a percent of each other on the 15360x8640 image; 100 and more lose the gain).
constexpr int kSplitMinSeqs = 1536;
constexpr uint32_t kHandoff = 48u;
// Inter-sequence kernel: a workgroup with at most this many boundaries to decode from walks them with the whole
// wavefront, one after the other (the walk takes about half the time of a lane's loop per subsequence).
constexpr int kInterCoopMax = 2;

JPGD_HD bool lut_esc(uint32_t e) { return e >= 0x8000u; }
JPGD_HD uint32_t lut_total(uint32_t e) { return e & 31u; }
JPGD_HD uint32_t lut_size(uint32_t e) { return (e >> 5) & 15u; }
JPGD_HD uint32_t lut_adv(uint32_t e) { return (e >> 9) & 63u; }
JPGD_HD uint32_t lut_esc_bits(uint32_t e) { return e & 7u; }
JPGD_HD uint32_t lut_esc_offset(uint32_t e) { return ((e >> 3) & 255u) << 1; }

// ---- s_info (paper, Section 4.1): one 16-byte record per subsequence --------------------------
//  x : decoder state after the last symbol that starts inside the subsequence
//        bits 0..5   p - (i+1)*L  (bit position relative to the end of the subsequence, 0..31)
//        bits 6..11  z            (zig-zag index of the next coefficient)
//        bits 12..15 u            (data unit inside the MCU)
//  y : bits 0..30: data units completed by the symbols that start inside the subsequence; bit 31: one of
//      those symbols was the first of a restart interval (the DC sums below then start at that symbol).
//      The paper's count n (zig-zag slots covered) is 64*units + z_i - z_{i-1}; keeping units and z apart
//      makes the exclusive scan deliver the output position as (unit index, z) without overflow.
//  z : sum of DC differences of component 0 (low 16 bits) and component 1 (high 16 bits), wrapped
//  w : the same for component 2 (low 16 bits)
struct SInfo {
    uint32_t x, y, z, w;
};

JPGD_HD uint32_t rec_units(uint32_t y) { return y & 0x7FFFFFFFu; }
JPGD_HD uint32_t rec_restarted(uint32_t y) { return y >> 31; }

JPGD_HD uint32_t pack_state(uint32_t p_rel, uint32_t z, uint32_t u) { return (p_rel & 63u) | (z << 6) | (u << 12); }
JPGD_HD uint32_t state_prel(uint32_t x) { return x & 63u; }
JPGD_HD uint32_t state_z(uint32_t x) { return (x >> 6) & 63u; }
JPGD_HD uint32_t state_u(uint32_t x) { return (x >> 12) & 15u; }

// ---- per-image descriptor, built on the host and uploaded with every call ----------------------
struct ImgDesc {
    // input
    uint64_t scan_off;     // byte offset of the stuffed scan inside d_scans (multiple of 16)
    uint32_t scan_bytes;   // stuffed length
    uint32_t tile0;        // first unstuff tile of this image
    uint32_t ntiles;
    // unstuffed stream
    uint64_t stream_off;   // byte offset inside the workspace's stream region (multiple of 256)
    // decomposition (upper bounds from the stuffed size; the true counts live in ImgState)
    uint32_t sub0;         // first s_info record of this image
    uint32_t nsub_max;
    uint32_t seq0;         // first workgroup of the intra-sequence kernel
    uint32_t nseq_max;
    uint32_t grp0;         // first workgroup of the scan/write kernels (groups of kWG subsequences)
    uint32_t ngrp_max;
    uint32_t bnd0;         // first workgroup of the inter-sequence kernel (64 boundaries each)
    uint32_t nbnd_wg;
    // scan syntax
    uint32_t total_units;
    uint32_t upm;          // data units per MCU
    uint32_t sched_dc;     // 4 bits per unit u: LUT slot of its DC table
    uint32_t sched_ac;     //                     ... of its AC table
    uint32_t sched_comp;   //                     component of unit u
    uint32_t lut_off;      // element (uint16) offset of this image's tables inside the LUT region
    uint32_t nslots;       // tables this image uses
    // output
    uint64_t coef_off;     // element offset into d_coef
    uint64_t pix_off;      // byte offset into d_pixels
    uint32_t width, height, ncomp;
    uint32_t hs, vs;       // luma sampling factors
    uint32_t mcus_x, mcus_y;
    uint32_t pix_wg0;      // first workgroup of the pixel kernel
    uint32_t pix_runs;     // workgroups per MCU row
    uint32_t qt_off;       // element (uint16) offset of 3 x 64 quantisation values (per component, zig-zag)
    // restart intervals (0 = the scan has none)
    uint32_t restart;      // MCUs per interval
    uint32_t nint;         // intervals in the scan
    uint32_t bmap_off;     // word offset of this image's interval-start bitmap (one bit per unstuffed byte,
                           // 128 words per unstuff tile plus 128 of slack)
    uint32_t ndc;          // DC tables of this image: slots 0 .. ndc-1; its AC tables follow, AC table k with pair bytes k
    uint32_t pad_;
};

// written by the unstuff kernels
struct ImgState {
    uint32_t nbytes;   // unstuffed length B
    uint32_t nsub;     // ceil(8B / L)
    uint32_t markers;  // restart markers met (counted by the unstuff kernels; must be nint - 1)
    uint32_t pad_;
};

// status word bits (device -> host)
constexpr uint32_t kStMismatch = 1u;   // a write lane did not end in the state recorded for its subsequence
constexpr uint32_t kStInvalid = 2u;    // write pass met bits that are no codeword, or a run past slot 63
constexpr uint32_t kStShort = 4u;      // stream ended before all data units were decoded
constexpr uint32_t kStUnit = 8u;       // unit index and recorded data-unit phase disagree

struct Status {
    uint32_t flags;
    uint32_t inter_changed;  // boundaries whose first comparison failed in the last inter-sequence round
    uint32_t pending;        // set if some sequence's records do not continue the state the sequence before it ends in
    uint32_t pad;
};

// write kernel: from this many bits of stream per data unit on, a workgroup's lanes lay down their own zeros instead
// of the workgroup clearing its stretch of the output first
constexpr uint32_t kDenseBitsPerUnit = 256u;
constexpr int kUnstuffTile = 4096;  // bytes per workgroup of the unstuff kernels (256 lanes x 16 bytes)
constexpr int kPixBlocks = 48;      // data units per workgroup of the pixel kernel
constexpr int kPixBlocksScaled = 192;  // ... of the reduced-size pixel kernels (a unit needs 16, 4 or 1 floats of LDS there)

JPGD_HD uint32_t align_up(uint32_t v, uint32_t a) { return (v + a - 1) / a * a; }

}  // namespace jpgd
