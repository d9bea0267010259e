/*
 * Baseline JPEG encoder used ONLY to manufacture seeded synthetic inputs
 * (the paper's photo/video-frame datasets are not redistributable, so every
 * test and benchmark input is produced here from a seeded pixel array).
 *
 * It follows the nine encoding steps the paper lists in its Section 2
 * ("JPEG Encoding and Decoding"): colour conversion, chroma subsampling,
 * 8x8 decomposition, forward DCT, quantisation, differential DC coding,
 * zig-zag, run-length coding, Huffman coding.  It is not part of the decoder
 * and not part of the decoder's CPU oracle: it shares no code, table or
 * header with either of them.
 *
 * Build: gcc -O2 -shared -fPIC -o libwl_jpeg_encoder.so jpeg_encoder.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ tables */

/* Quantisation matrices of ITU-T T.81 Annex K.1 (row-major, natural order). */
static const uint8_t k_base_luma[64] = {
    16, 11, 10, 16, 24,  40,  51,  61,
    12, 12, 14, 19, 26,  58,  60,  55,
    14, 13, 16, 24, 40,  57,  69,  56,
    14, 17, 22, 29, 51,  87,  80,  62,
    18, 22, 37, 56, 68,  109, 103, 77,
    24, 35, 55, 64, 81,  104, 113, 92,
    49, 64, 78, 87, 103, 121, 120, 101,
    72, 92, 95, 98, 112, 100, 103, 99};
static const uint8_t k_base_chroma[64] = {
    17, 18, 24, 47, 99, 99, 99, 99,
    18, 21, 26, 66, 99, 99, 99, 99,
    24, 26, 56, 99, 99, 99, 99, 99,
    47, 66, 99, 99, 99, 99, 99, 99,
    99, 99, 99, 99, 99, 99, 99, 99,
    99, 99, 99, 99, 99, 99, 99, 99,
    99, 99, 99, 99, 99, 99, 99, 99,
    99, 99, 99, 99, 99, 99, 99, 99};

/* Typical Huffman tables of ITU-T T.81 Annex K.3 (BITS / HUFFVAL lists). */
static const uint8_t k_dc_luma_bits[16] = {0, 1, 5, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0};
static const uint8_t k_dc_chroma_bits[16] = {0, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0, 0};
static const uint8_t k_dc_vals[12] = {0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11};
static const uint8_t k_ac_luma_bits[16] = {0, 2, 1, 3, 3, 2, 4, 3, 5, 5, 4, 4, 0, 0, 1, 125};
static const uint8_t k_ac_luma_vals[162] = {
    0x01, 0x02, 0x03, 0x00, 0x04, 0x11, 0x05, 0x12, 0x21, 0x31, 0x41, 0x06, 0x13, 0x51, 0x61, 0x07,
    0x22, 0x71, 0x14, 0x32, 0x81, 0x91, 0xA1, 0x08, 0x23, 0x42, 0xB1, 0xC1, 0x15, 0x52, 0xD1, 0xF0,
    0x24, 0x33, 0x62, 0x72, 0x82, 0x09, 0x0A, 0x16, 0x17, 0x18, 0x19, 0x1A, 0x25, 0x26, 0x27, 0x28,
    0x29, 0x2A, 0x34, 0x35, 0x36, 0x37, 0x38, 0x39, 0x3A, 0x43, 0x44, 0x45, 0x46, 0x47, 0x48, 0x49,
    0x4A, 0x53, 0x54, 0x55, 0x56, 0x57, 0x58, 0x59, 0x5A, 0x63, 0x64, 0x65, 0x66, 0x67, 0x68, 0x69,
    0x6A, 0x73, 0x74, 0x75, 0x76, 0x77, 0x78, 0x79, 0x7A, 0x83, 0x84, 0x85, 0x86, 0x87, 0x88, 0x89,
    0x8A, 0x92, 0x93, 0x94, 0x95, 0x96, 0x97, 0x98, 0x99, 0x9A, 0xA2, 0xA3, 0xA4, 0xA5, 0xA6, 0xA7,
    0xA8, 0xA9, 0xAA, 0xB2, 0xB3, 0xB4, 0xB5, 0xB6, 0xB7, 0xB8, 0xB9, 0xBA, 0xC2, 0xC3, 0xC4, 0xC5,
    0xC6, 0xC7, 0xC8, 0xC9, 0xCA, 0xD2, 0xD3, 0xD4, 0xD5, 0xD6, 0xD7, 0xD8, 0xD9, 0xDA, 0xE1, 0xE2,
    0xE3, 0xE4, 0xE5, 0xE6, 0xE7, 0xE8, 0xE9, 0xEA, 0xF1, 0xF2, 0xF3, 0xF4, 0xF5, 0xF6, 0xF7, 0xF8,
    0xF9, 0xFA};
static const uint8_t k_ac_chroma_bits[16] = {0, 2, 1, 2, 4, 4, 3, 4, 7, 5, 4, 4, 0, 1, 2, 119};
static const uint8_t k_ac_chroma_vals[162] = {
    0x00, 0x01, 0x02, 0x03, 0x11, 0x04, 0x05, 0x21, 0x31, 0x06, 0x12, 0x41, 0x51, 0x07, 0x61, 0x71,
    0x13, 0x22, 0x32, 0x81, 0x08, 0x14, 0x42, 0x91, 0xA1, 0xB1, 0xC1, 0x09, 0x23, 0x33, 0x52, 0xF0,
    0x15, 0x62, 0x72, 0xD1, 0x0A, 0x16, 0x24, 0x34, 0xE1, 0x25, 0xF1, 0x17, 0x18, 0x19, 0x1A, 0x26,
    0x27, 0x28, 0x29, 0x2A, 0x35, 0x36, 0x37, 0x38, 0x39, 0x3A, 0x43, 0x44, 0x45, 0x46, 0x47, 0x48,
    0x49, 0x4A, 0x53, 0x54, 0x55, 0x56, 0x57, 0x58, 0x59, 0x5A, 0x63, 0x64, 0x65, 0x66, 0x67, 0x68,
    0x69, 0x6A, 0x73, 0x74, 0x75, 0x76, 0x77, 0x78, 0x79, 0x7A, 0x82, 0x83, 0x84, 0x85, 0x86, 0x87,
    0x88, 0x89, 0x8A, 0x92, 0x93, 0x94, 0x95, 0x96, 0x97, 0x98, 0x99, 0x9A, 0xA2, 0xA3, 0xA4, 0xA5,
    0xA6, 0xA7, 0xA8, 0xA9, 0xAA, 0xB2, 0xB3, 0xB4, 0xB5, 0xB6, 0xB7, 0xB8, 0xB9, 0xBA, 0xC2, 0xC3,
    0xC4, 0xC5, 0xC6, 0xC7, 0xC8, 0xC9, 0xCA, 0xD2, 0xD3, 0xD4, 0xD5, 0xD6, 0xD7, 0xD8, 0xD9, 0xDA,
    0xE2, 0xE3, 0xE4, 0xE5, 0xE6, 0xE7, 0xE8, 0xE9, 0xEA, 0xF2, 0xF3, 0xF4, 0xF5, 0xF6, 0xF7, 0xF8,
    0xF9, 0xFA};

/* scan position -> natural (row*8+col) index, produced by walking the
 * anti-diagonals of the 8x8 matrix in alternating direction */
static uint8_t g_scan_to_natural[64];
static double g_cos[8][8]; /* g_cos[k][n] = c(k)/2 * cos((2n+1) k pi / 16) */
static int g_ready = 0;

static void init_constants(void) {
    if (g_ready) return;
    int idx = 0;
    for (int d = 0; d < 15; ++d) {
        /* cells on anti-diagonal d have row+col == d */
        int lo = d < 8 ? 0 : d - 7, hi = d < 8 ? d : 7;
        if (d & 1) { /* odd diagonals run downwards: row increasing */
            for (int r = lo; r <= hi; ++r) g_scan_to_natural[idx++] = (uint8_t)(r * 8 + (d - r));
        } else { /* even diagonals run upwards: row decreasing */
            for (int r = hi; r >= lo; --r) g_scan_to_natural[idx++] = (uint8_t)(r * 8 + (d - r));
        }
    }
    const double pi = 3.14159265358979323846;
    for (int k = 0; k < 8; ++k)
        for (int n = 0; n < 8; ++n)
            g_cos[k][n] = (k == 0 ? sqrt(0.5) : 1.0) * 0.5 * cos((2 * n + 1) * k * pi / 16.0);
    g_ready = 1;
}

/* ------------------------------------------------------------ byte output */

typedef struct {
    uint8_t* data;
    size_t len, cap;
    uint64_t acc; /* pending bits, right aligned */
    int nacc;
} sink_t;

static void sink_byte(sink_t* s, uint8_t b) {
    if (s->len == s->cap) {
        s->cap = s->cap ? s->cap * 2 : 1 << 16;
        s->data = (uint8_t*)realloc(s->data, s->cap);
    }
    s->data[s->len++] = b;
}
static void sink_u16(sink_t* s, unsigned v) {
    sink_byte(s, (uint8_t)(v >> 8));
    sink_byte(s, (uint8_t)v);
}
/* entropy-coded bits, most significant bit first, with 0x00 stuffed after 0xFF */
static void sink_bits(sink_t* s, unsigned code, int nbits) {
    if (nbits == 0) return;
    s->acc = (s->acc << nbits) | (code & ((1u << nbits) - 1u));
    s->nacc += nbits;
    while (s->nacc >= 8) {
        uint8_t b = (uint8_t)(s->acc >> (s->nacc - 8));
        sink_byte(s, b);
        if (b == 0xFF) sink_byte(s, 0x00);
        s->nacc -= 8;
    }
}
static void sink_flush_ones(sink_t* s) {
    if (s->nacc > 0) {
        int pad = 8 - s->nacc;
        sink_bits(s, (1u << pad) - 1u, pad);
    }
}

/* -------------------------------------------------------- Huffman tables */

typedef struct {
    uint8_t bits[16];
    uint8_t vals[256];
    int nvals;
    uint16_t code[256];
    uint8_t size[256]; /* 0 = symbol has no code */
} hufftab_t;

/* canonical code assignment: shortest first, in list order, counting upward */
static void assign_codes(hufftab_t* t) {
    memset(t->size, 0, sizeof t->size);
    memset(t->code, 0, sizeof t->code);
    unsigned next = 0;
    int k = 0;
    for (int len = 1; len <= 16; ++len) {
        for (int i = 0; i < t->bits[len - 1]; ++i, ++k) {
            t->code[t->vals[k]] = (uint16_t)next++;
            t->size[t->vals[k]] = (uint8_t)len;
        }
        next <<= 1;
    }
    t->nvals = k;
}

static void set_table(hufftab_t* t, const uint8_t* bits, const uint8_t* vals, int n) {
    memcpy(t->bits, bits, 16);
    memset(t->vals, 0, sizeof t->vals);
    memcpy(t->vals, vals, (size_t)n);
    assign_codes(t);
}

/*
 * Per-image optimised table from symbol counts (procedure of T.81 Annex K.2):
 * an extra never-used symbol takes the place of the all-ones codeword; code
 * lengths come from repeatedly merging the two rarest groups; lengths above
 * 16 are shortened by moving pairs of leaves up the tree.
 */
static void build_optimal_table(hufftab_t* t, const uint64_t* freq_in) {
    uint64_t freq[257];
    int len[257], link[257];
    for (int i = 0; i < 256; ++i) freq[i] = freq_in[i];
    freq[256] = 1;
    for (int i = 0; i < 257; ++i) { len[i] = 0; link[i] = -1; }
    for (;;) {
        int a = -1, b = -1; /* a = rarest, b = second rarest; ties -> larger index */
        for (int i = 0; i < 257; ++i)
            if (freq[i] && (a < 0 || freq[i] <= freq[a])) a = i;
        for (int i = 0; i < 257; ++i)
            if (freq[i] && i != a && (b < 0 || freq[i] <= freq[b])) b = i;
        if (b < 0) break;
        freq[a] += freq[b];
        freq[b] = 0;
        /* every leaf in both chains gets one level deeper; append chain b to chain a */
        int i = a;
        for (;;) { len[i]++; if (link[i] < 0) break; i = link[i]; }
        link[i] = b;
        for (i = b; i >= 0; i = link[i]) len[i]++;
    }
    int count[260];
    memset(count, 0, sizeof count);
    for (int i = 0; i < 257; ++i)
        if (len[i]) count[len[i]]++;
    for (int l = 257; l > 16; --l) {
        while (count[l] > 0) {
            int j = l - 2;
            while (count[j] == 0) --j;
            count[l] -= 2;     /* two deepest siblings: one moves up to the parent level ... */
            count[l - 1] += 1;
            count[j + 1] += 2; /* ... the other shares a split leaf taken from level j */
            count[j] -= 1;
        }
    }
    int l = 16;
    while (count[l] == 0) --l;
    count[l]--; /* drop the reserved pseudo symbol (it has the longest code) */
    for (int i = 0; i < 16; ++i) t->bits[i] = (uint8_t)count[i + 1];
    /* symbols by increasing original code length, then by symbol value */
    int k = 0;
    memset(t->vals, 0, sizeof t->vals);
    for (int ll = 1; ll <= 257; ++ll)
        for (int s = 0; s < 256; ++s)
            if (len[s] == ll) t->vals[k++] = (uint8_t)s;
    assign_codes(t);
}

/* ------------------------------------------------------------- transform */

static void fdct8x8(const double in[64], double out[64]) {
    double tmp[64];
    for (int y = 0; y < 8; ++y) /* rows: horizontal frequency u */
        for (int u = 0; u < 8; ++u) {
            double s = 0;
            for (int x = 0; x < 8; ++x) s += in[y * 8 + x] * g_cos[u][x];
            tmp[y * 8 + u] = s;
        }
    for (int u = 0; u < 8; ++u) /* columns: vertical frequency v */
        for (int v = 0; v < 8; ++v) {
            double s = 0;
            for (int y = 0; y < 8; ++y) s += tmp[y * 8 + u] * g_cos[v][y];
            out[v * 8 + u] = s;
        }
}

static int magnitude_category(int v) {
    int a = v < 0 ? -v : v, n = 0;
    while (a) { ++n; a >>= 1; }
    return n;
}

/* ---------------------------------------------------------------- encoder */

typedef struct {
    int width, height, ncomp;
    int hs, vs; /* luma sampling factors (chroma is 1x1) */
    int mcus_x, mcus_y, units_per_mcu;
    uint16_t qt[2][64]; /* natural order */
} enc_geom_t;

static void make_qtable(const uint8_t* base, int quality, uint16_t* out) {
    if (quality < 1) quality = 1;
    if (quality > 100) quality = 100;
    int scale = quality < 50 ? 5000 / quality : 200 - 2 * quality;
    for (int i = 0; i < 64; ++i) {
        int q = (base[i] * scale + 50) / 100;
        if (q < 1) q = 1;
        if (q > 255) q = 255;
        out[i] = (uint16_t)q;
    }
}

/* sample of component c (0=Y,1=Cb,2=Cr) at pixel (x,y), coordinates clamped to the image
 * (edge replication for incomplete MCUs, Section 2 of the paper) */
static double comp_sample(const uint8_t* px, const enc_geom_t* g, int c, int x, int y) {
    if (x >= g->width) x = g->width - 1;
    if (y >= g->height) y = g->height - 1;
    if (g->ncomp == 1) return px[(size_t)y * g->width + x];
    const uint8_t* p = px + ((size_t)y * g->width + x) * 3;
    double r = p[0], gg = p[1], b = p[2];
    if (c == 0) return 0.299 * r + 0.587 * gg + 0.114 * b;
    if (c == 1) return -0.168736 * r - 0.331264 * gg + 0.5 * b + 128.0;
    return 0.5 * r - 0.418688 * gg - 0.081312 * b + 128.0;
}

/* quantised coefficients of every data unit in scan (MCU-interleaved) order,
 * zig-zag order inside a unit, DC stored as the absolute value */
static void transform_all(const uint8_t* px, const enc_geom_t* g, int16_t* coef) {
    size_t k = 0;
    double blk[64], freq[64];
    for (int my = 0; my < g->mcus_y; ++my)
        for (int mx = 0; mx < g->mcus_x; ++mx)
            for (int c = 0; c < g->ncomp; ++c) {
                int nh = c == 0 ? g->hs : 1, nv = c == 0 ? g->vs : 1;
                int sx = c == 0 ? 1 : g->hs, sy = c == 0 ? 1 : g->vs; /* subsampling step */
                const uint16_t* q = g->qt[c == 0 ? 0 : 1];
                for (int by = 0; by < nv; ++by)
                    for (int bx = 0; bx < nh; ++bx, ++k) {
                        /* top-left of this unit in component-plane coordinates */
                        int cx0 = (mx * nh + bx) * 8, cy0 = (my * nv + by) * 8;
                        for (int y = 0; y < 8; ++y)
                            for (int x = 0; x < 8; ++x) {
                                double s = 0;
                                for (int dy = 0; dy < sy; ++dy)
                                    for (int dx = 0; dx < sx; ++dx)
                                        s += comp_sample(px, g, c, (cx0 + x) * sx + dx, (cy0 + y) * sy + dy);
                                blk[y * 8 + x] = s / (sx * sy) - 128.0;
                            }
                        fdct8x8(blk, freq);
                        for (int i = 0; i < 64; ++i) {
                            int nat = g_scan_to_natural[i];
                            double t = freq[nat] / q[nat];
                            long v = (long)(t < 0 ? -floor(-t + 0.5) : floor(t + 0.5));
                            long lim = i == 0 ? 1024 : 1023;
                            if (v > lim) v = lim;
                            if (v < -lim) v = -lim;
                            coef[k * 64 + i] = (int16_t)v;
                        }
                    }
            }
}

typedef void (*emit_fn)(void* ctx, int table_class, int table_id, int symbol, unsigned extra, int nextra);

/* walks all data units and reports every (Huffman symbol, extra bits) pair */
static void scan_symbols(const enc_geom_t* g, const int16_t* coef, int restart_interval, emit_fn emit,
                         void (*restart)(void*, int), void* ctx) {
    int pred[3] = {0, 0, 0};
    size_t k = 0;
    long mcu = 0, total = (long)g->mcus_x * g->mcus_y;
    int rst = 0;
    for (; mcu < total; ++mcu) {
        if (restart_interval && mcu && mcu % restart_interval == 0) {
            restart(ctx, rst);
            rst = (rst + 1) & 7;
            pred[0] = pred[1] = pred[2] = 0;
        }
        for (int c = 0; c < g->ncomp; ++c) {
            int n = c == 0 ? g->hs * g->vs : 1, tid = c == 0 ? 0 : 1;
            for (int b = 0; b < n; ++b, ++k) {
                const int16_t* blk = coef + k * 64;
                int diff = blk[0] - pred[c];
                pred[c] = blk[0];
                int cat = magnitude_category(diff);
                unsigned bitsv = diff >= 0 ? (unsigned)diff : (unsigned)(diff + (1 << cat) - 1);
                emit(ctx, 0, tid, cat, bitsv, cat);
                int run = 0;
                for (int i = 1; i < 64; ++i) {
                    int v = blk[i];
                    if (v == 0) { ++run; continue; }
                    while (run > 15) { emit(ctx, 1, tid, 0xF0, 0, 0); run -= 16; }
                    cat = magnitude_category(v);
                    bitsv = v >= 0 ? (unsigned)v : (unsigned)(v + (1 << cat) - 1);
                    emit(ctx, 1, tid, (run << 4) | cat, bitsv, cat);
                    run = 0;
                }
                if (run) emit(ctx, 1, tid, 0x00, 0, 0);
            }
        }
    }
}

typedef struct { uint64_t freq[2][2][256]; } count_ctx_t;
static void count_emit(void* c, int cls, int tid, int sym, unsigned e, int ne) {
    (void)e; (void)ne;
    ((count_ctx_t*)c)->freq[cls][tid][sym]++;
}
static void count_restart(void* c, int n) { (void)c; (void)n; }

typedef struct { sink_t* s; hufftab_t (*tab)[2]; } write_ctx_t;
static void write_emit(void* c, int cls, int tid, int sym, unsigned e, int ne) {
    write_ctx_t* w = (write_ctx_t*)c;
    hufftab_t* t = &w->tab[cls][tid];
    sink_bits(w->s, t->code[sym], t->size[sym]);
    sink_bits(w->s, e, ne);
}
static void write_restart(void* c, int n) {
    write_ctx_t* w = (write_ctx_t*)c;
    sink_flush_ones(w->s);
    sink_byte(w->s, 0xFF);
    sink_byte(w->s, (uint8_t)(0xD0 + n));
}

static void put_dht(sink_t* s, int cls, int id, const hufftab_t* t) {
    sink_u16(s, 0xFFC4);
    sink_u16(s, (unsigned)(2 + 1 + 16 + t->nvals));
    sink_byte(s, (uint8_t)((cls << 4) | id));
    for (int i = 0; i < 16; ++i) sink_byte(s, t->bits[i]);
    for (int i = 0; i < t->nvals; ++i) sink_byte(s, t->vals[i]);
}

/*
 * pixels : gray (ncomp=1, H*W) or interleaved RGB (ncomp=3, H*W*3), uint8
 * subsampling : 0 = 4:4:4, 1 = 4:2:2 (luma 2x1), 2 = 4:2:0 (luma 2x2); ignored for gray
 * optimize : 0 = Annex K tables, 1 = per-image tables built from symbol counts
 * restart_interval : MCUs between RSTn markers, 0 = none
 * out_file/out_len : malloc'ed file, release with wl_free
 * out_coef : if not NULL, receives 64*total_units int16 quantised coefficients
 *            (scan order, zig-zag inside a unit, absolute DC)
 * scan_offset/scan_len : if not NULL, position and length of the entropy-coded bytes
 * returns 0, or -1 on bad arguments
 */
int wl_encode_jpeg(const uint8_t* pixels, int width, int height, int ncomp, int subsampling, int quality,
                   int optimize, int restart_interval, uint8_t** out_file, size_t* out_len, int16_t* out_coef,
                   size_t* scan_offset, size_t* scan_len) {
    if (!pixels || width < 1 || height < 1 || width > 65535 || height > 65535) return -1;
    if (ncomp != 1 && ncomp != 3) return -1;
    if (subsampling < 0 || subsampling > 2) return -1;
    init_constants();
    enc_geom_t g;
    g.width = width; g.height = height; g.ncomp = ncomp;
    g.hs = (ncomp == 3 && subsampling >= 1) ? 2 : 1;
    g.vs = (ncomp == 3 && subsampling == 2) ? 2 : 1;
    g.mcus_x = (width + 8 * g.hs - 1) / (8 * g.hs);
    g.mcus_y = (height + 8 * g.vs - 1) / (8 * g.vs);
    g.units_per_mcu = ncomp == 1 ? 1 : g.hs * g.vs + 2;
    make_qtable(k_base_luma, quality, g.qt[0]);
    make_qtable(k_base_chroma, quality, g.qt[1]);

    size_t units = (size_t)g.mcus_x * g.mcus_y * g.units_per_mcu;
    int16_t* coef = out_coef ? out_coef : (int16_t*)malloc(units * 64 * sizeof(int16_t));
    if (!coef) return -1;
    transform_all(pixels, &g, coef);

    hufftab_t tab[2][2]; /* [class: 0 DC, 1 AC][id: 0 luma, 1 chroma] */
    if (optimize) {
        count_ctx_t* cc = (count_ctx_t*)calloc(1, sizeof *cc);
        scan_symbols(&g, coef, restart_interval, count_emit, count_restart, cc);
        for (int cls = 0; cls < 2; ++cls)
            for (int id = 0; id < (ncomp == 3 ? 2 : 1); ++id) build_optimal_table(&tab[cls][id], cc->freq[cls][id]);
        free(cc);
    } else {
        set_table(&tab[0][0], k_dc_luma_bits, k_dc_vals, 12);
        set_table(&tab[0][1], k_dc_chroma_bits, k_dc_vals, 12);
        set_table(&tab[1][0], k_ac_luma_bits, k_ac_luma_vals, 162);
        set_table(&tab[1][1], k_ac_chroma_bits, k_ac_chroma_vals, 162);
    }

    sink_t s;
    memset(&s, 0, sizeof s);
    sink_u16(&s, 0xFFD8);
    /* JFIF APP0 */
    sink_u16(&s, 0xFFE0); sink_u16(&s, 16);
    sink_byte(&s, 'J'); sink_byte(&s, 'F'); sink_byte(&s, 'I'); sink_byte(&s, 'F'); sink_byte(&s, 0);
    sink_u16(&s, 0x0101); sink_byte(&s, 0); sink_u16(&s, 1); sink_u16(&s, 1); sink_byte(&s, 0); sink_byte(&s, 0);
    for (int id = 0; id < (ncomp == 3 ? 2 : 1); ++id) {
        sink_u16(&s, 0xFFDB); sink_u16(&s, 67); sink_byte(&s, (uint8_t)id);
        for (int i = 0; i < 64; ++i) sink_byte(&s, (uint8_t)g.qt[id][g_scan_to_natural[i]]);
    }
    sink_u16(&s, 0xFFC0); sink_u16(&s, (unsigned)(8 + 3 * ncomp)); sink_byte(&s, 8);
    sink_u16(&s, (unsigned)height); sink_u16(&s, (unsigned)width); sink_byte(&s, (uint8_t)ncomp);
    for (int c = 0; c < ncomp; ++c) {
        sink_byte(&s, (uint8_t)(c + 1));
        sink_byte(&s, (uint8_t)(c == 0 ? (g.hs << 4) | g.vs : 0x11));
        sink_byte(&s, (uint8_t)(c == 0 ? 0 : 1));
    }
    for (int id = 0; id < (ncomp == 3 ? 2 : 1); ++id) {
        put_dht(&s, 0, id, &tab[0][id]);
        put_dht(&s, 1, id, &tab[1][id]);
    }
    if (restart_interval) { sink_u16(&s, 0xFFDD); sink_u16(&s, 4); sink_u16(&s, (unsigned)restart_interval); }
    sink_u16(&s, 0xFFDA); sink_u16(&s, (unsigned)(6 + 2 * ncomp)); sink_byte(&s, (uint8_t)ncomp);
    for (int c = 0; c < ncomp; ++c) {
        sink_byte(&s, (uint8_t)(c + 1));
        sink_byte(&s, (uint8_t)(c == 0 ? 0x00 : 0x11));
    }
    sink_byte(&s, 0); sink_byte(&s, 63); sink_byte(&s, 0);
    size_t scan_begin = s.len;
    write_ctx_t w;
    w.s = &s; w.tab = tab;
    scan_symbols(&g, coef, restart_interval, write_emit, write_restart, &w);
    sink_flush_ones(&s);
    if (scan_offset) *scan_offset = scan_begin;
    if (scan_len) *scan_len = s.len - scan_begin;
    sink_u16(&s, 0xFFD9);
    if (!out_coef) free(coef);
    *out_file = s.data;
    *out_len = s.len;
    return 0;
}

void wl_free(void* p) { free(p); }

/* Annex K tables and the quality scaling, exported so tests can compare them with an outside encoder's headers */
void wl_quant_table(int chroma, int quality, uint16_t out_natural[64]) {
    make_qtable(chroma ? k_base_chroma : k_base_luma, quality, out_natural);
}
void wl_scan_order(uint8_t out[64]) {
    init_constants();
    memcpy(out, g_scan_to_natural, 64);
}
