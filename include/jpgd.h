/*
 * jpgd -- baseline-JPEG decoding on one AMD MI355X (gfx950) with the
 * self-synchronising parallel Huffman decoder of Weissenberger & Schmidt,
 * "Accelerating JPEG Decompression on GPUs" (arXiv 2111.09219).
 *
 * C ABI.  Every function returns JPGD_OK (0) or a negative jpgd_status; none
 * aborts or throws.  Pointers marked [host] are ordinary host memory, pointers
 * marked [device] are HIP device memory on the current device.  The library
 * never allocates or frees device memory: the caller (PyTorch in the Python
 * binding) owns every device buffer and the stream.
 *
 * Pipeline behind jpgd_decode / jpgd_decode_batch (paper, Section 4,
 * Algorithm 1), all of it in HIP kernels:
 *   unstuff       drop the 0x00 after every 0xFF of the entropy-coded bytes
 *                 (the paper does not mention byte stuffing; a baseline stream
 *                 cannot be cut into fixed-size subsequences without it)
 *   sync (intra)  Algorithm 3, first loop: one lane per subsequence, own decode
 *                 (Algorithm 2) then overflow into the neighbours until the
 *                 decoder state (bit position, data unit, zig-zag index) matches
 *   sync (inter)  Algorithm 3, second loop: one lane per sequence boundary
 *   scan          Algorithm 1, exclusive prefix sum over s_info.n, here over
 *                 (completed data units, DC-difference sums per component)
 *   write         Algorithm 1 last loop / Algorithm 2 with write=true: re-decode
 *                 from the true state and scatter coefficients; run/EOB expansion
 *   DC            Section 4.2: per-component prefix sum of DC differences
 *                 (carried through the scan above; see jpgd_decode)
 *   pixels        Section 4.3: de-zigzag, dequantise, 8x8 IDCT; plus MCU ->
 *                 image placement, chroma replication and YCbCr -> RGB
 */
#ifndef JPGD_H
#define JPGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    JPGD_OK = 0,
    JPGD_E_ARG = -1,         /* NULL pointer, bad size, bad config value                     */
    JPGD_E_TRUNCATED = -2,   /* file or segment ends early, no end-of-image marker            */
    JPGD_E_MARKER = -3,      /* not a JPEG, marker syntax broken, scan before frame header    */
    JPGD_E_UNSUPPORTED = -4, /* valid JPEG outside the supported subset (see jpgd_parse)      */
    JPGD_E_TABLE = -5,       /* missing or malformed Huffman / quantisation table             */
    JPGD_E_CORRUPT = -6,     /* entropy-coded data inconsistent with the headers              */
    JPGD_E_WORKSPACE = -7,   /* workspace too small or misaligned                             */
    JPGD_E_HIP = -8,         /* a HIP runtime call failed                                     */
    JPGD_E_BUSY = -9         /* too many calls in flight (jpgd_decode_batch_async without jpgd_wait) */
} jpgd_status;

/*
 * Everything the decoder needs from the headers of one file.  Plain data,
 * filled by jpgd_parse, owned by the caller, never holds pointers.
 */
typedef struct {
    uint32_t width, height;       /* pixels                                                          */
    uint32_t ncomp;               /* 1 (grayscale) or 3 (YCbCr)                                      */
    uint8_t hsamp[3], vsamp[3];   /* sampling factors per component                                  */
    uint8_t tq[3], td[3], ta[3];  /* quantisation / DC / AC table ids per component                  */
    uint16_t qt[4][64];           /* quantisation tables in the order stored in the file (zig-zag)   */
    uint8_t qt_present[4];
    uint8_t dht_bits[2][4][16];   /* [0 = DC, 1 = AC][table id]: number of codes of length 1..16     */
    uint8_t dht_vals[2][4][256];  /* symbols in order of increasing code                             */
    uint8_t dht_present[2][4];
    uint32_t mcu_w, mcu_h;        /* pixels per MCU: 8x8, 16x8 or 16x16 (paper, Section 2)           */
    uint32_t mcus_x, mcus_y;
    uint32_t units_per_mcu;       /* 1, 3, 4 or 6 data units                                         */
    uint32_t total_units;         /* data units (8x8 blocks) in the scan                             */
    uint64_t scan_offset;         /* first entropy-coded byte inside the file                        */
    uint64_t scan_bytes;          /* entropy-coded bytes, still byte-stuffed, up to the EOI marker   */
    uint32_t restart_interval;    /* MCUs per restart interval (DRI); 0 = the scan has no markers    */
} jpgd_info;

typedef struct {
    uint32_t subseq_bits;  /* subsequence size in bits ("s*32" in Algorithm 1): 128, 256, 512, 1024
                              or 2048; 0 = choose per call from the size of the streams and their
                              bits per data unit                                                 */
    uint32_t overlap;      /* subsequences by which neighbouring sequences overlap (warm-up lanes
                              in front of each sequence); 0 = the paper's disjoint sequences;
                              must be < 192; 0xFFFFFFFF = library default (16 or 32)               */
    uint32_t max_rounds;   /* upper bound on inter-sequence synchronisation rounds; 0 = number of
                              sequences (always enough)                                             */
    uint32_t flags;        /* JPGD_F_*: at most one of the JPGD_F_SCALE_* */
    uint32_t timing_mask;  /* bit k set: bracket kernel k (JPGD_K_*) with HIP events on the stream
                              and report its duration; 0 = no events                               */
    uint32_t sync_split;   /* intra-sequence synchronisation (Algorithm 3, first loop) in one kernel or in
                              two (the second one takes over when few chains of a sequence are left and
                              runs them without the LDS copy of the stream, so that a CU holds more
                              sequences): 0 = the library decides (two for calls with many more sequences
                              than the chip holds at a time), 1 = one kernel, 2 = two kernels wherever
                              the call allows it (no restart intervals, at most four tables per image).
                              The result does not depend on it.                                     */
} jpgd_config;

#define JPGD_F_NO_PIXELS 1u /* stop after the coefficients even if a pixel buffer is given */
#define JPGD_F_PLANAR 2u    /* d_pixels receives the component planes instead of interleaved RGB: the paper's own
                               output (Section 3: one array per colour channel; Section 4.3: the IDCT is the last
                               step).  Per image, at pixel_offsets[i]: the luma plane (height x width), then, for
                               3 components, Cb and Cr, each ceil(height / v) x ceil(width / h) for luma sampling
                               factors h x v; samples rounded once and clamped, no upsampling, no colour
                               conversion.  The planes never take more than height x width x ncomp bytes. */

#define JPGD_F_SCALE_2 4u   /* d_pixels receives the image at 1/2 of its size: ceil(width / 2) x ceil(height / 2) pixels
                               (with JPGD_F_PLANAR: every plane at ceil(plane size / 2)).  Of every data unit the 4 x 4
                               lowest frequencies go through the 4-point inverse transform of the same family as the
                               8-point one of Section 4.3 (same factor, so a flat unit keeps its value); all later
                               steps as at full size.  The coefficients are always delivered in full.  For callers
                               that want a smaller image than the file holds: the paper names the inverse transform
                               as the stage that limits its decoder (Section 6), and this output skips most of it. */
#define JPGD_F_SCALE_4 8u   /* the same at 1/4: 2 x 2 lowest frequencies, 2-point transform */
#define JPGD_F_SCALE_8 12u  /* the same at 1/8: one sample per data unit, DC * Q / 8 + 128 */

/* kernels of the pipeline, in launch order */
enum {
    JPGD_K_UNSTUFF_COUNT = 0, /* unstuff: bytes to drop per tile                                   */
    JPGD_K_UNSTUFF_SCAN,      /* unstuff: exclusive scan of the tile counts, unstuffed length      */
    JPGD_K_UNSTUFF_SCATTER,   /* unstuff: compaction                                               */
    JPGD_K_SYNC_INTRA,        /* Algorithm 3, first loop                                           */
    JPGD_K_SYNC_TAIL,         /* Algorithm 3, first loop: its late rounds, when run as a kernel of their own */
    JPGD_K_SYNC_INTER,        /* Algorithm 3, second loop                                          */
    JPGD_K_SCAN_TOTALS,       /* exclusive scan over s_info: totals per group of 256 records       */
    JPGD_K_SCAN_PREFIX,       /* exclusive scan over s_info: prefix of the group totals            */
    JPGD_K_WRITE,             /* Algorithm 1, write pass                                           */
    JPGD_K_PIXELS,            /* Section 4.3 plus colour                                           */
    JPGD_N_KERNELS
};

/* What a decode call did; filled on return (host memory). */
typedef struct {
    uint32_t subseq_bits;   /* subsequence size used                                              */
    uint32_t n_subseq;      /* subsequences over all images (upper bound from the stuffed sizes)  */
    uint32_t n_sequences;   /* thread blocks of the intra-sequence kernel                         */
    uint32_t inter_rounds;  /* inter-sequence rounds run                                          */
    uint32_t redo;          /* further rounds (inter-sequence + totals kernels) it took until every
                               sequence continued the state the one before it ends in; the write pass
                               and the pixels then ran a second time                               */
    uint32_t device_flags;  /* raw status word from the device                                    */
    uint32_t launches[JPGD_N_KERNELS];  /* launches of each kernel in this call                          */
    float kernel_ms[JPGD_N_KERNELS];    /* summed duration of the launches selected by timing_mask       */
} jpgd_report;

/*
 * Host only, touches no GPU.  Reads the marker segments of a baseline JPEG
 * file (paper, Section 4.1: the batch is parsed and the Huffman tables are
 * extracted on the host before any kernel runs) and locates the entropy-coded segment without
 * scanning it: it ends at the last EOI marker of the file.
 *
 * Accepted: SOF0, 8-bit, one scan, 1 component or 3 components with chroma
 * sampled 1x1 and luma 1x1, 2x1, 1x2 or 2x2; with or without restart
 * intervals (DRI / RSTm).
 * JPGD_E_UNSUPPORTED: progressive / extended / lossless / arithmetic frames,
 * 12-bit, other component counts or sampling, several scans.
 * JPGD_E_TABLE: table id > 3, more than 256 symbols, more codes of some
 * length than that length can hold, a DC table with a symbol above 11 (a DC
 * symbol is a number of value bits; 8-bit samples need at most 11), a table a
 * component refers to missing.
 * JPGD_E_TRUNCATED / JPGD_E_MARKER: as named.
 */
int jpgd_parse(const uint8_t* file /*[host]*/, size_t len, jpgd_info* out /*[host]*/);

/*
 * Bytes of device workspace jpgd_decode_batch needs for these images and this
 * config (0 on bad arguments): the unstuffed streams, s_info with one record per
 * subsequence (paper, Section 4.1; Algorithm 1 allocates it per call), the
 * tables and the partial results of the scans.  The workspace must be 256-byte aligned.  Its
 * contents need not be preserved between calls and may be uninitialised.
 */
size_t jpgd_workspace_bytes(const jpgd_info* infos /*[host]*/, int n_images, const jpgd_config* cfg /*[host], may be NULL*/);

/*
 * Decodes n images in one go (paper, Algorithm 1, "batched").
 *
 *  infos          [host]   n parsed headers
 *  d_scans        [device] the entropy-coded bytes of all images (still byte-stuffed, without the
 *                          EOI marker); image i occupies scan_offsets[i] .. + infos[i].scan_bytes;
 *                          16-byte aligned.  The kernels read whole 16-byte words: the bytes up to
 *                          the next multiple of 16 after each scan must be readable (their content
 *                          is ignored; device allocations are granular enough that this only
 *                          matters for a scan placed at the very end of a sub-allocated block)
 *  scan_offsets   [host]   n byte offsets into d_scans, each a multiple of 16
 *  d_coef         [device] int16 output, 16-byte aligned, may not be NULL; image i gets 64*total_units
 *                          values at element offset coef_offsets[i] (must be a multiple of 64):
 *                          data units in scan (MCU-interleaved) order, zig-zag order inside a
 *                          unit, quantised (not dequantised), DC un-differenced
 *  coef_offsets   [host]
 *  d_pixels       [device] uint8 output or NULL: image i at byte offset pixel_offsets[i],
 *                          height x width x ncomp interleaved (gray or RGB), cropped to the
 *                          true size (other layouts and sizes: JPGD_F_PLANAR, JPGD_F_SCALE_*)
 *  pixel_offsets  [host]   may be NULL iff d_pixels is NULL
 *  d_workspace    [device] jpgd_workspace_bytes(...) bytes, 256-byte aligned
 *  cfg            [host]   may be NULL for defaults
 *  stream                  a hipStream_t (as void*); NULL = the default stream
 *  report         [host]   may be NULL
 *
 * All work is enqueued on `stream`.  The call returns once the device's
 * verdict has arrived (every lane of the write pass checks that it ends in
 * the state recorded for its subsequence): the verdict decides whether further
 * synchronisation rounds are needed and is the source of JPGD_E_CORRUPT.  At
 * that point d_coef is complete; the kernel that fills d_pixels may still be
 * running, so d_pixels is complete in stream order like the output of any
 * kernel: work enqueued on `stream` afterwards sees it, a host that reads it
 * synchronises the stream first.  Calls from several threads, or several calls
 * in flight (jpgd_decode_batch_async), do not wait for each other inside the
 * library; each needs a workspace and outputs of its own.
 * On JPGD_E_CORRUPT the outputs hold unspecified values but nothing outside
 * them has been written.
 *
 * DC: the per-component prefix sum of Section 4.2 is computed hierarchically
 * -- per-subsequence sums of DC differences during synchronisation, their
 * exclusive scan together with the unit counts, and a running sum in the write
 * pass -- so d_coef is written exactly once, with absolute DC values.
 */
int jpgd_decode_batch(int n, const jpgd_info* infos, const uint8_t* d_scans, const uint64_t* scan_offsets,
                      int16_t* d_coef, const uint64_t* coef_offsets, uint8_t* d_pixels,
                      const uint64_t* pixel_offsets, void* d_workspace, size_t workspace_bytes,
                      const jpgd_config* cfg, void* stream, jpgd_report* report);

/*
 * The same call in two halves, for the end-to-end setting the paper times (Section 5, experimental setup:
 * the transfer of the compressed data is part of the measured time, so a decoder that is fed batch after batch
 * has to overlap the copy of the next batch with the decoding of this one).
 *
 * jpgd_decode_batch_async validates, builds the per-call tables and enqueues every kernel of the path on
 * `stream`, then returns without waiting for the GPU; *call receives a handle.  infos and the offset arrays may be
 * freed as soon as it returns; the device buffers and the workspace belong to the call until jpgd_wait returns.
 * Several calls may be in flight at once, on the same stream or on different ones (at most 64: JPGD_E_BUSY),
 * each with its own workspace and outputs.
 *
 * jpgd_wait blocks until the call's verdict has arrived, runs the further synchronisation rounds in the rare case
 * that they are needed (it may therefore enqueue more work on the call's stream), fills *report (may be NULL)
 * and releases the handle, whatever it returns.  Its return value is that of jpgd_decode_batch.  Every handle
 * must be waited for exactly once, by any thread.
 * jpgd_decode_batch is the one followed by the other.
 */
typedef struct jpgd_call jpgd_call;
int jpgd_decode_batch_async(int n, const jpgd_info* infos, const uint8_t* d_scans, const uint64_t* scan_offsets,
                            int16_t* d_coef, const uint64_t* coef_offsets, uint8_t* d_pixels,
                            const uint64_t* pixel_offsets, void* d_workspace, size_t workspace_bytes,
                            const jpgd_config* cfg, void* stream, jpgd_call** call /*[host]*/);
int jpgd_wait(jpgd_call* call, jpgd_report* report /*[host], may be NULL*/);

/* One image: jpgd_decode_batch with n = 1 and all offsets 0. */
int jpgd_decode(const jpgd_info* info, const uint8_t* d_scan, int16_t* d_coef, uint8_t* d_pixels,
                void* d_workspace, size_t workspace_bytes, const jpgd_config* cfg, void* stream,
                jpgd_report* report);

/*
 * For callers that cannot allocate: code between hipStreamBeginCapture and hipStreamEndCapture, serving loops
 * with a fixed memory budget, harnesses that forbid hipMalloc.  jpgd_decode_static is jpgd_decode without the
 * workspace argument: the workspace is an array of JPGD_STATIC_WORKSPACE_BYTES inside the library's device image
 * (every GPU the library runs on holds one copy until the process ends), and the pinned parameter block was set
 * up by jpgd_init.  It calls no hipMalloc, hipHostMalloc, hipFree or any other allocating routine, creates no
 * events and changes no function attribute.
 *
 * jpgd_init: once per device, with that device current, before the first jpgd_decode_static there (calling it
 * again is harmless).  It looks up the array's device address, allocates the pinned parameter and verdict blocks
 * of the fixed slot and asks for the kernels' dynamic LDS.  Not needed by the other entry points.
 *
 * jpgd_decode_static: arguments as jpgd_decode.  JPGD_E_WORKSPACE if the image needs more workspace than the
 * array holds (jpgd_workspace_bytes(info, 1, cfg) > JPGD_STATIC_WORKSPACE_BYTES: roughly, scans beyond 1.8 MB),
 * JPGD_E_ARG if jpgd_init has not run on the current device or cfg->timing_mask is not 0.  Results are those of
 * jpgd_decode.  All calls on one GPU share that GPU's array and the library lets them take turns: a second call
 * blocks until the first has returned; the array keeps the last call's contents, and nothing in it has to be
 * cleared by the caller.  Like jpgd_decode it returns when the verdict has arrived.
 */
#define JPGD_STATIC_WORKSPACE_BYTES (4u << 20)
int jpgd_init(void);
size_t jpgd_static_workspace_bytes(void);
int jpgd_decode_static(const jpgd_info* info, const uint8_t* d_scan, int16_t* d_coef, uint8_t* d_pixels,
                       const jpgd_config* cfg, void* stream, jpgd_report* report);

/*
 * Stage-level entry points (used by the tests to check single steps against the oracle).
 *
 * jpgd_unstuff: the byte-unstuffing step alone.  d_in (16-byte aligned, n bytes, readable up to the
 * next multiple of 16) is compacted into
 * d_out (256-byte aligned, room for n + 256 bytes: the kernel clears 192 bytes after the last one);
 * *out_len [host] receives the unstuffed length.  d_workspace: 256-byte aligned, at least
 * 1024 + 4 * ceil(n / 4096) bytes.  Returns after the stream has drained.  The input is taken as a scan
 * without restart intervals: only stuffed zeros are dropped (the decode calls, which know a file's DRI, also
 * drop the RSTm markers).
 */
int jpgd_unstuff(const uint8_t* d_in /*[device]*/, size_t n, uint8_t* d_out /*[device]*/, size_t* out_len /*[host]*/,
                 void* d_workspace, size_t workspace_bytes, void* stream);

/*
 * Copies the synchronisation result (paper, Section 4.1: the array s_info once
 * Algorithm 3 has run) of the most recent decode call that used
 * this workspace to the host: for image `image`, subsequence i < *n_subseq,
 *   p[i]      bit position (unstuffed stream) of the first symbol starting at or after (i+1)*subseq_bits
 *   u[i],z[i] data unit inside the MCU and zig-zag index at that point
 *   units[i]  bits 0..30: data units completed by symbols starting inside subsequence i;
 *             bit 31: one of those symbols was the first of a restart interval
 *   dcsum[3*i+c] sum of DC differences of component c among those symbols (as int16, wrapped),
 *             counted from the last symbol that began a restart interval, if there was one
 * Arrays must have room for `capacity` entries; JPGD_E_ARG if fewer than needed.
 */
int jpgd_read_sync_info(const void* d_workspace, int image, uint32_t capacity, uint32_t* n_subseq,
                        uint64_t* p, uint32_t* u, uint32_t* z, uint32_t* units, int32_t* dcsum, void* stream);

const char* jpgd_strerror(int status);

/* ABI version of this header: bumped on any incompatible change. */
int jpgd_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* JPGD_H */
