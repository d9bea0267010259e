/*
 * CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, sequential, deliberately slow baseline-JPEG decoder.  It defines
 * what the GPU decoder must produce and is called only from tests/, from
 * __graft_entry__.smoke() and from bench.py's cpu_baseline leg.  It shares no
 * code, header, table or helper with the GPU path or with the encoder that
 * manufactures inputs.
 *
 * Why a sequential decoder is the right oracle: the paper's method (Section 4,
 * Algorithms 1-3) only finds, in parallel, the decoder state at which each
 * subsequence has to be entered; once a lane's state equals the sequential
 * decoder's state, everything it decodes is what the sequential decoder
 * decodes (Section 3, discussion of Table I).  The coefficients are therefore
 * exactly those of the plain decode written out here, in the order of the
 * format description in Section 2 of the paper:
 *
 *   Huffman decoding + run-length expansion   (Section 2, last paragraphs)
 *   DC difference decoding                    (Section 2, P = DC_i - DC_{i-1}; Section 4.2)
 *   zig-zag reordering, dequantisation, IDCT  (Section 4.3)
 *   MCU -> image placement                    (Section 2 MCU layout; Section 4.3 last paragraph)
 *   chroma upsampling and YCbCr -> RGB        (not in the paper: replicate + JFIF matrix, in double,
 *                                              one rounding at the very end)
 *
 * Floating point is double throughout.  Nothing here is tuned.
 *
 * Pins (tests/test_oracle_*.py): the worked example of Table I; closed-form
 * streams; canonical-code invariants; an independent encoder's coefficients;
 * Pillow-written files; scipy's inverse DCT; DC-only blocks.
 *
 * Build: gcc -O2 -shared -fPIC -o liborc_jpeg.so jpeg_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
    ORC_OK = 0,
    ORC_E_ARG = -1,
    ORC_E_TRUNCATED = -2,
    ORC_E_MARKER = -3,
    ORC_E_UNSUPPORTED = -4,
    ORC_E_TABLE = -5,
    ORC_E_CORRUPT = -6
};

typedef struct {
    int present;
    uint8_t bits[16];  /* number of codes of length 1..16 */
    uint8_t vals[256]; /* symbols in code order */
    int nvals;
    /* canonical code bookkeeping per length (index 1..16) */
    int32_t mincode[17], maxcode[17], valptr[17];
} orc_huff;

typedef struct {
    int32_t width, height, ncomp;
    int32_t hs[3], vs[3];     /* sampling factors per component */
    int32_t tq[3], td[3], ta[3];
    int32_t hmax, vmax;
    int32_t mcus_x, mcus_y, units_per_mcu;
    int64_t total_units;
    int64_t scan_offset, scan_len; /* entropy-coded bytes inside the file, still stuffed */
    int32_t restart_interval;
    uint16_t qt[4][64]; /* in the order stored in the file (zig-zag) */
    int32_t qt_present[4];
} orc_info;

typedef struct {
    orc_info info;
    orc_huff huff[2][4]; /* [0 = DC, 1 = AC][table id] */
    const uint8_t* file;
    size_t file_len;
    /* data unit u of an MCU belongs to component unit_comp[u] and sits at (unit_bx, unit_by) inside it */
    int unit_comp[10], unit_bx[10], unit_by[10];
} orc_image;

/* ------------------------------------------------------------------ header */

static int build_huff(orc_huff* h) {
    int total = 0;
    for (int i = 0; i < 16; ++i) total += h->bits[i];
    if (total > 256) return ORC_E_TABLE;
    h->nvals = total;
    int32_t code = 0;
    int k = 0;
    for (int len = 1; len <= 16; ++len) {
        int n = h->bits[len - 1];
        h->valptr[len] = k;
        h->mincode[len] = code;
        h->maxcode[len] = n ? code + n - 1 : -1;
        code += n;
        k += n;
        if (code > (1 << len)) return ORC_E_TABLE; /* more codes than the length can hold */
        code <<= 1;
    }
    return ORC_OK;
}

static int rd16(const uint8_t* p) { return (p[0] << 8) | p[1]; }

int orc_open(const uint8_t* file, size_t len, orc_image** out) {
    if (!file || !out) return ORC_E_ARG;
    if (len < 4 || file[0] != 0xFF || file[1] != 0xD8) return ORC_E_MARKER;
    orc_image* im = (orc_image*)calloc(1, sizeof *im);
    if (!im) return ORC_E_ARG;
    im->file = file;
    im->file_len = len;
    size_t pos = 2;
    int have_sof = 0, rc = ORC_OK;
    for (;;) {
        if (pos + 4 > len) { rc = ORC_E_TRUNCATED; break; }
        if (file[pos] != 0xFF) { rc = ORC_E_MARKER; break; }
        int m = file[pos + 1];
        if (m == 0xFF) { ++pos; continue; } /* fill byte */
        if (m == 0xD8 || m == 0x01 || (m >= 0xD0 && m <= 0xD7)) { pos += 2; continue; }
        if (m == 0xD9) { rc = ORC_E_MARKER; break; } /* end of image before any scan */
        int seglen = rd16(file + pos + 2);
        if (seglen < 2 || pos + 2 + (size_t)seglen > len) { rc = ORC_E_TRUNCATED; break; }
        const uint8_t* seg = file + pos + 4;
        int n = seglen - 2;
        if (m == 0xC0) {
            if (have_sof) { rc = ORC_E_UNSUPPORTED; break; }
            if (n < 6) { rc = ORC_E_TRUNCATED; break; }
            if (seg[0] != 8) { rc = ORC_E_UNSUPPORTED; break; }
            im->info.height = rd16(seg + 1);
            im->info.width = rd16(seg + 3);
            im->info.ncomp = seg[5];
            if (im->info.ncomp != 1 && im->info.ncomp != 3) { rc = ORC_E_UNSUPPORTED; break; }
            if (n < 6 + 3 * im->info.ncomp) { rc = ORC_E_TRUNCATED; break; }
            if (im->info.width == 0 || im->info.height == 0) { rc = ORC_E_UNSUPPORTED; break; }
            for (int c = 0; c < im->info.ncomp; ++c) {
                im->info.hs[c] = seg[7 + 3 * c] >> 4;
                im->info.vs[c] = seg[7 + 3 * c] & 15;
                im->info.tq[c] = seg[8 + 3 * c];
                if (im->info.tq[c] > 3) { rc = ORC_E_TABLE; break; }
            }
            if (rc) break;
            have_sof = 1;
        } else if ((m >= 0xC1 && m <= 0xCF) && m != 0xC4 && m != 0xC8) {
            rc = ORC_E_UNSUPPORTED; /* extended, progressive, lossless, arithmetic */
            break;
        } else if (m == 0xC4) {
            int q = 0;
            while (q < n) {
                if (q + 17 > n) { rc = ORC_E_TRUNCATED; break; }
                int cls = seg[q] >> 4, id = seg[q] & 15;
                if (cls > 1 || id > 3) { rc = ORC_E_TABLE; break; }
                orc_huff* h = &im->huff[cls][id];
                memset(h, 0, sizeof *h);
                memcpy(h->bits, seg + q + 1, 16);
                int total = 0;
                for (int i = 0; i < 16; ++i) total += h->bits[i];
                if (total > 256) { rc = ORC_E_TABLE; break; }
                if (q + 17 + total > n) { rc = ORC_E_TRUNCATED; break; }
                memcpy(h->vals, seg + q + 17, (size_t)total);
                rc = build_huff(h);
                if (rc) break;
                h->present = 1;
                q += 17 + total;
            }
            if (rc) break;
        } else if (m == 0xDB) {
            int q = 0;
            while (q < n) {
                int prec = seg[q] >> 4, id = seg[q] & 15;
                if (id > 3 || prec > 1) { rc = ORC_E_TABLE; break; }
                int need = 1 + (prec ? 128 : 64);
                if (q + need > n) { rc = ORC_E_TRUNCATED; break; }
                for (int i = 0; i < 64; ++i)
                    im->info.qt[id][i] = prec ? (uint16_t)rd16(seg + q + 1 + 2 * i) : seg[q + 1 + i];
                im->info.qt_present[id] = 1;
                q += need;
            }
            if (rc) break;
        } else if (m == 0xDD) {
            if (n < 2) { rc = ORC_E_TRUNCATED; break; }
            im->info.restart_interval = rd16(seg);
        } else if (m == 0xDA) {
            if (!have_sof) { rc = ORC_E_MARKER; break; }
            if (n < 1 || seg[0] != im->info.ncomp) { rc = ORC_E_UNSUPPORTED; break; } /* one interleaved scan only */
            if (n < 1 + 2 * im->info.ncomp + 3) { rc = ORC_E_TRUNCATED; break; }
            for (int c = 0; c < im->info.ncomp; ++c) {
                im->info.td[c] = seg[2 + 2 * c] >> 4;
                im->info.ta[c] = seg[2 + 2 * c] & 15;
                if (im->info.td[c] > 3 || im->info.ta[c] > 3) { rc = ORC_E_TABLE; break; }
            }
            if (rc) break;
            im->info.scan_offset = (int64_t)(pos + 2 + (size_t)seglen);
            break;
        }
        pos += 2 + (size_t)seglen;
    }
    if (!rc) {
        orc_info* in = &im->info;
        if (in->ncomp == 1) { in->hs[0] = in->vs[0] = 1; } /* a single component is never interleaved */
        in->hmax = in->vmax = 1;
        for (int c = 0; c < in->ncomp; ++c) {
            if (in->hs[c] < 1 || in->vs[c] < 1) rc = ORC_E_UNSUPPORTED;
            if (in->hs[c] > in->hmax) in->hmax = in->hs[c];
            if (in->vs[c] > in->vmax) in->vmax = in->vs[c];
        }
        if (in->ncomp == 3) {
            int ok = in->hs[1] == 1 && in->vs[1] == 1 && in->hs[2] == 1 && in->vs[2] == 1 &&
                     (in->hs[0] == 1 || in->hs[0] == 2) && (in->vs[0] == 1 || in->vs[0] == 2);
            if (!ok) rc = ORC_E_UNSUPPORTED;
        }
    }
    if (!rc) {
        orc_info* in = &im->info;
        in->mcus_x = (in->width + 8 * in->hmax - 1) / (8 * in->hmax);
        in->mcus_y = (in->height + 8 * in->vmax - 1) / (8 * in->vmax);
        int u = 0;
        for (int c = 0; c < in->ncomp; ++c)
            for (int by = 0; by < in->vs[c]; ++by)
                for (int bx = 0; bx < in->hs[c]; ++bx) {
                    im->unit_comp[u] = c;
                    im->unit_bx[u] = bx;
                    im->unit_by[u] = by;
                    ++u;
                }
        in->units_per_mcu = u;
        in->total_units = (int64_t)in->mcus_x * in->mcus_y * u;
        for (int c = 0; c < in->ncomp; ++c) {
            if (!in->qt_present[in->tq[c]]) rc = ORC_E_TABLE;
            if (!im->huff[0][in->td[c]].present || !im->huff[1][in->ta[c]].present) rc = ORC_E_TABLE;
        }
    }
    if (!rc) {
        /* the entropy-coded segment runs up to the next marker that is neither a stuffed zero nor, when a
         * restart interval is defined, a restart marker RST0..RST7 */
        size_t p = (size_t)im->info.scan_offset;
        int ri = im->info.restart_interval != 0;
        while (p + 1 < len &&
               !(file[p] == 0xFF && file[p + 1] != 0x00 && !(ri && file[p + 1] >= 0xD0 && file[p + 1] <= 0xD7)))
            ++p;
        if (p + 1 >= len) rc = ORC_E_TRUNCATED;
        else if (file[p + 1] != 0xD9) rc = ORC_E_UNSUPPORTED; /* further scans, stray markers */
        im->info.scan_len = (int64_t)p - im->info.scan_offset;
    }
    if (rc) { free(im); return rc; }
    *out = im;
    return ORC_OK;
}

void orc_close(orc_image* im) { free(im); }

int orc_get_info(const orc_image* im, orc_info* out) {
    if (!im || !out) return ORC_E_ARG;
    *out = im->info;
    return ORC_OK;
}

/* raw table lists, for tests of the canonical-code invariants */
int orc_get_huffman(const orc_image* im, int cls, int id, uint8_t bits[16], uint8_t vals[256]) {
    if (!im || cls < 0 || cls > 1 || id < 0 || id > 3 || !im->huff[cls][id].present) return ORC_E_ARG;
    memcpy(bits, im->huff[cls][id].bits, 16);
    memcpy(vals, im->huff[cls][id].vals, 256);
    return im->huff[cls][id].nvals;
}

/* codeword of every symbol as (code, length); length 0 = symbol absent */
int orc_get_codes(const orc_image* im, int cls, int id, uint16_t code[256], uint8_t length[256]) {
    if (!im || cls < 0 || cls > 1 || id < 0 || id > 3 || !im->huff[cls][id].present) return ORC_E_ARG;
    const orc_huff* h = &im->huff[cls][id];
    memset(code, 0, 512);
    memset(length, 0, 256);
    for (int len = 1; len <= 16; ++len)
        for (int i = 0; i < h->bits[len - 1]; ++i) {
            int sym = h->vals[h->valptr[len] + i];
            code[sym] = (uint16_t)(h->mincode[len] + i);
            length[sym] = (uint8_t)len;
        }
    return ORC_OK;
}

/* -------------------------------------------------------------- unstuffing */

/* removes the 0x00 that follows every 0xFF; out may be NULL to get the length only */
int64_t orc_unstuff_bytes(const uint8_t* in, int64_t n, uint8_t* out) {
    int64_t k = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (out) out[k] = in[i];
        ++k;
        if (in[i] == 0xFF && i + 1 < n && in[i + 1] == 0x00) ++i;
    }
    return k;
}

/*
 * The same for a segment with restart markers (T.81 E.1.4 / F.1.2.3: every Ri MCUs the encoder pads the
 * last byte with 1-bits and emits RSTm, m = 0..7 in turn; the decoder discards the padding, checks the
 * marker and resets the DC predictors).  Stuffed zeros and the two bytes of every RSTm are removed;
 * starts[k] receives the offset, in the output, of the first byte of restart interval k (starts[0] = 0).
 * Returns the output length, or -1 if the markers do not count 0,1,..7,0,.. or there are more than
 * max_starts intervals.  out and starts may be NULL.
 */
int64_t orc_unstuff_restart(const uint8_t* in, int64_t n, uint8_t* out, int64_t* starts, int64_t max_starts,
                            int64_t* nstarts) {
    int64_t k = 0, ns = 1;
    if (starts && max_starts > 0) starts[0] = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (in[i] == 0xFF && i + 1 < n && in[i + 1] >= 0xD0 && in[i + 1] <= 0xD7) {
            if ((in[i + 1] & 7) != ((ns - 1) & 7)) return -1;
            if (starts) {
                if (ns >= max_starts) return -1;
                starts[ns] = k;
            }
            ++ns;
            ++i;
            continue;
        }
        if (out) out[k] = in[i];
        ++k;
        if (in[i] == 0xFF && i + 1 < n && in[i + 1] == 0x00) ++i;
    }
    if (nstarts) *nstarts = ns;
    return k;
}

/* ---------------------------------------------------------- entropy decode */

typedef struct {
    const uint8_t* data; /* unstuffed */
    int64_t nbits;       /* bits available */
    int64_t pos;         /* next bit */
    int overrun;
} bitrd;

static int next_bit(bitrd* r) {
    if (r->pos >= r->nbits) { r->overrun = 1; r->pos++; return 0; }
    int b = (r->data[r->pos >> 3] >> (7 - (r->pos & 7))) & 1;
    r->pos++;
    return b;
}

static int read_bits(bitrd* r, int n) {
    int v = 0;
    for (int i = 0; i < n; ++i) v = (v << 1) | next_bit(r);
    return v;
}

/* one Huffman symbol, read bit by bit against the canonical code ranges.
 * returns the symbol, or -1 when 16 bits match no codeword (then exactly one bit has been consumed) */
static int read_symbol(bitrd* r, const orc_huff* h) {
    int64_t start = r->pos;
    int32_t code = 0;
    for (int len = 1; len <= 16; ++len) {
        code = (code << 1) | next_bit(r);
        if (h->maxcode[len] >= 0 && code >= h->mincode[len] && code <= h->maxcode[len])
            return h->vals[h->valptr[len] + (code - h->mincode[len])];
    }
    r->pos = start + 1;
    return -1;
}

/* value bits -> signed coefficient ("signed ones' complement", Section 2) */
static int extend(int v, int nbits) {
    if (nbits == 0) return 0;
    return v >= (1 << (nbits - 1)) ? v : v - ((1 << nbits) - 1);
}

/* One syntax element as the paper's decode_next_symbol() (Algorithm 2) sees it. */
typedef struct {
    int64_t p;    /* bit position where it starts */
    int u, z;     /* data unit inside the MCU and zig-zag index before it */
    int is_dc;
    int run;      /* zeros preceding the coefficient (15 for ZRL, 63-z for EOB) */
    int size;     /* number of value bits */
    int value;    /* decoded coefficient (DC: the difference); 0 for ZRL/EOB */
    int kind;     /* 0 coefficient, 1 ZRL, 2 EOB, 3 no codeword matched */
    int length;   /* bits consumed */
} orc_symbol;

/* decoder state (p, u, z): bit position, data unit inside the MCU, zig-zag index */
typedef struct { int64_t p; int u, z; } orc_state;

/*
 * Decodes the syntax element at state *s and advances *s past it.
 * DC table when z == 0, else the AC table of the unit's component (Section 4.1).
 * Rules where the paper is silent (they matter only for decoders that are not yet
 * synchronised, or corrupt input): no matching codeword -> consume one bit, state
 * otherwise unchanged; AC symbol with zero size and run not in {0,15} -> end of block;
 * z running past 63 -> unit complete.
 */
static void step(const orc_image* im, bitrd* r, orc_state* s, orc_symbol* sym) {
    const orc_info* in = &im->info;
    int c = im->unit_comp[s->u];
    r->pos = s->p;
    sym->p = s->p; sym->u = s->u; sym->z = s->z;
    sym->is_dc = s->z == 0;
    sym->run = 0; sym->size = 0; sym->value = 0; sym->kind = 0;
    int advance; /* zig-zag slots covered */
    if (s->z == 0) {
        int t = read_symbol(r, &im->huff[0][in->td[c]]);
        if (t < 0) { sym->kind = 3; sym->length = 1; s->p += 1; return; }
        sym->size = t > 16 ? 16 : t; /* DC symbols are plain sizes; valid streams use 0..11 */
        sym->value = extend(read_bits(r, sym->size), sym->size);
        advance = 1;
    } else {
        int rs = read_symbol(r, &im->huff[1][in->ta[c]]);
        if (rs < 0) { sym->kind = 3; sym->length = 1; s->p += 1; return; }
        int run = rs >> 4, size = rs & 15;
        if (size == 0) {
            if (run == 15) { sym->kind = 1; sym->run = 15; advance = 16; }
            else { sym->kind = 2; sym->run = 63 - s->z; advance = 64 - s->z; }
        } else {
            sym->run = run;
            sym->size = size;
            sym->value = extend(read_bits(r, size), size);
            advance = run + 1;
        }
    }
    sym->length = (int)(r->pos - s->p);
    s->p = r->pos;
    s->z += advance;
    if (s->z >= 64) {
        s->z = 0;
        s->u = (s->u + 1) % in->units_per_mcu;
    }
}

/* number of restart intervals of the scan (1 without DRI) */
static int64_t interval_count(const orc_image* im) {
    const orc_info* in = &im->info;
    if (in->restart_interval == 0) return 1;
    int64_t mcus = (int64_t)in->mcus_x * in->mcus_y;
    return (mcus + in->restart_interval - 1) / in->restart_interval;
}

/* unstuffed stream (markers removed) and, if starts != NULL, the byte offset of every restart interval */
static int unstuffed_scan(const orc_image* im, uint8_t** buf, int64_t* nbytes, int64_t** starts) {
    const uint8_t* src = im->file + im->info.scan_offset;
    int64_t nint = interval_count(im);
    int64_t* st = (int64_t*)malloc((size_t)nint * sizeof(int64_t));
    if (!st) return ORC_E_ARG;
    int64_t found = 0;
    int64_t n = orc_unstuff_restart(src, im->info.scan_len, NULL, NULL, 0, &found);
    if (n < 0 || found != nint) { free(st); return ORC_E_CORRUPT; } /* wrong number or order of markers */
    uint8_t* b = (uint8_t*)malloc((size_t)n + 8);
    if (!b) { free(st); return ORC_E_ARG; }
    orc_unstuff_restart(src, im->info.scan_len, b, st, nint, &found);
    memset(b + n, 0, 8);
    *buf = b;
    *nbytes = n;
    if (starts) *starts = st; else free(st);
    return ORC_OK;
}

int64_t orc_unstuffed_len(const orc_image* im) {
    return orc_unstuff_restart(im->file + im->info.scan_offset, im->info.scan_len, NULL, NULL, 0, NULL);
}
int orc_unstuff(const orc_image* im, uint8_t* out) {
    return orc_unstuff_restart(im->file + im->info.scan_offset, im->info.scan_len, out, NULL, 0, NULL) < 0 ? ORC_E_CORRUPT
                                                                                                       : ORC_OK;
}
int64_t orc_interval_count(const orc_image* im) { return interval_count(im); }
/* byte offsets of the restart intervals in the unstuffed stream; starts has room for orc_interval_count() */
int orc_interval_starts(const orc_image* im, int64_t* starts) {
    int64_t found = 0;
    int64_t n = orc_unstuff_restart(im->file + im->info.scan_offset, im->info.scan_len, NULL, starts, interval_count(im),
                                    &found);
    return (n < 0 || found != interval_count(im)) ? ORC_E_CORRUPT : ORC_OK;
}

/*
 * End of a restart interval: the decoder stands at bit *p after the interval's last symbol; what is left of
 * that byte must be 1-bits (at most 7), and decoding continues at the first bit of the next interval.
 */
static int enter_interval(const uint8_t* buf, int64_t* p, int64_t start_byte) {
    int64_t target = start_byte * 8;
    if (*p > target || target - *p > 7) return ORC_E_CORRUPT;
    for (int64_t b = *p; b < target; ++b)
        if (!((buf[b >> 3] >> (7 - (b & 7))) & 1)) return ORC_E_CORRUPT;
    *p = target;
    return ORC_OK;
}

/*
 * Quantised coefficients of all data units: coef[64*k + i], k in scan (MCU-interleaved)
 * order, i in zig-zag order, DC already un-differenced (predictor 0 at the image start,
 * one predictor per component).  end_bit (may be NULL) receives the bit position after
 * the last symbol.
 */
int orc_decode_coefficients(const orc_image* im, int16_t* coef, int64_t* end_bit) {
    if (!im || !coef) return ORC_E_ARG;
    uint8_t* buf;
    int64_t nbytes;
    int64_t* starts;
    int rc = unstuffed_scan(im, &buf, &nbytes, &starts);
    if (rc) return rc;
    bitrd r = {buf, nbytes * 8, 0, 0};
    const orc_info* in = &im->info;
    memset(coef, 0, (size_t)in->total_units * 64 * sizeof(int16_t));
    int32_t pred[3] = {0, 0, 0};
    orc_state s = {0, 0, 0};
    orc_symbol sym;
    const int64_t units_per_interval = (int64_t)in->restart_interval * in->units_per_mcu; /* 0: no restarts */
    for (int64_t k = 0; k < in->total_units && !rc; ++k) {
        if (units_per_interval && k > 0 && k % units_per_interval == 0) {
            /* a new restart interval: padding discarded, predictors back to zero */
            rc = enter_interval(buf, &s.p, starts[k / units_per_interval]);
            if (rc) break;
            pred[0] = pred[1] = pred[2] = 0;
        }
        int unit_u = s.u;
        for (;;) {
            int z_before = s.z;
            step(im, &r, &s, &sym);
            if (sym.kind == 3 || r.overrun) { rc = ORC_E_CORRUPT; break; }
            if (sym.is_dc) {
                int c = im->unit_comp[unit_u];
                pred[c] += sym.value;
                coef[k * 64] = (int16_t)pred[c];
            } else if (sym.kind == 0) {
                int at = z_before + sym.run;
                if (at > 63) { rc = ORC_E_CORRUPT; break; }
                coef[k * 64 + at] = (int16_t)sym.value;
            } else if (sym.kind == 1 && z_before + 16 > 64) {
                rc = ORC_E_CORRUPT;
                break;
            }
            if (s.z == 0) break; /* unit complete */
        }
    }
    if (end_bit) *end_bit = s.p;
    free(buf);
    free(starts);
    return rc;
}

/*
 * Syntax elements from an arbitrary bit position and decoder state, over an explicit
 * (already unstuffed) bit string: the experiment of Table I.  Stops after max_symbols
 * or when the next symbol would start at or beyond nbits.  Returns the count.
 */
int orc_trace(const orc_image* im, const uint8_t* bits, int64_t nbits, int64_t start_bit, int u, int z,
              orc_symbol* out, int max_symbols) {
    if (!im || !bits || !out || u < 0 || u >= im->info.units_per_mcu || z < 0 || z > 63) return ORC_E_ARG;
    bitrd r = {bits, nbits, 0, 0};
    orc_state s = {start_bit, u, z};
    int n = 0;
    while (n < max_symbols && s.p < nbits) step(im, &r, &s, &out[n++]);
    return n;
}

/*
 * True decoder state at every subsequence boundary, for subsequences of L bits of the
 * unstuffed stream (Section 4.1: the content s_info must have once synchronisation is
 * complete).  Entry i describes the sequential decoder at the first symbol that starts
 * at or after bit (i+1)*L:
 *   p[i], u[i], z[i]   its state there,
 *   units[i]           data units completed by symbols that start inside subsequence i,
 *   slots[i]           zig-zag slots those symbols cover (= 64*units[i] + z[i] - z[i-1]),
 *   dcsum[3*i + c]     sum of the DC differences of component c among them,
 *   restart[i]         1 if one of them is the first symbol of a restart interval other than the first;
 *                      dcsum then only counts symbols from the last such one on (the predictors were reset).
 * At the end of a restart interval the decoder moves to the first bit of the next interval at once, so a
 * state never points into padding.  Once all data units are decoded the state stays at the end position.
 * nsub must be ceil(8*unstuffed_len / L).
 */
int orc_boundary_states(const orc_image* im, int L, int64_t nsub, int64_t* p, int32_t* u, int32_t* z,
                        int32_t* units, int64_t* slots, int32_t* dcsum, int32_t* restart) {
    if (!im || L < 32 || nsub < 1) return ORC_E_ARG;
    uint8_t* buf;
    int64_t nbytes;
    int64_t* starts;
    int rc = unstuffed_scan(im, &buf, &nbytes, &starts);
    if (rc) return rc;
    bitrd r = {buf, nbytes * 8, 0, 0};
    const orc_info* in = &im->info;
    const int64_t units_per_interval = (int64_t)in->restart_interval * in->units_per_mcu;
    orc_state s = {0, 0, 0};
    orc_symbol sym;
    int64_t done = 0;
    int fresh = 0; /* the next symbol is the first of a restart interval (other than the image's first) */
    for (int64_t i = 0; i < nsub; ++i) {
        int64_t limit = (i + 1) * (int64_t)L;
        int32_t nu = 0, dc[3] = {0, 0, 0}, rs = 0;
        int64_t ns = 0;
        while (s.p < limit && done < in->total_units) {
            if (fresh) { rs = 1; dc[0] = dc[1] = dc[2] = 0; fresh = 0; }
            int zb = s.z, ub = s.u;
            step(im, &r, &s, &sym);
            if (sym.kind == 3 || r.overrun) { free(buf); free(starts); return ORC_E_CORRUPT; }
            if (sym.is_dc) dc[im->unit_comp[ub]] += sym.value;
            if (s.z == 0) {
                ++nu; ++done; ns += 64 - zb;
                if (units_per_interval && done < in->total_units && done % units_per_interval == 0) {
                    /* the interval is complete: the decoder moves on to the next one at once */
                    if (enter_interval(buf, &s.p, starts[done / units_per_interval])) {
                        free(buf); free(starts);
                        return ORC_E_CORRUPT;
                    }
                    fresh = 1;
                }
            } else {
                ns += s.z - zb;
            }
        }
        p[i] = s.p; u[i] = s.u; z[i] = s.z;
        units[i] = nu; slots[i] = ns;
        dcsum[3 * i] = dc[0]; dcsum[3 * i + 1] = dc[1]; dcsum[3 * i + 2] = dc[2];
        if (restart) restart[i] = rs;
    }
    free(buf);
    free(starts);
    return ORC_OK;
}

/* ------------------------------------------------------------------ pixels */

static double g_c[8][8]; /* g_c[x][u] = C(u) cos((2x+1) u pi / 16) */
static int g_zz[64];     /* zig-zag position -> row*8 + col */
static int g_init = 0;

static void init_tables(void) {
    if (g_init) return;
    const double pi = 3.14159265358979323846;
    for (int x = 0; x < 8; ++x)
        for (int u = 0; u < 8; ++u) g_c[x][u] = (u == 0 ? 1.0 / sqrt(2.0) : 1.0) * cos((2 * x + 1) * u * pi / 16.0);
    /* zig-zag: start at the top-left, move along anti-diagonals, turning at the matrix edges */
    int r = 0, c = 0;
    for (int i = 0; i < 64; ++i) {
        g_zz[i] = r * 8 + c;
        if ((r + c) % 2 == 0) { /* moving up-right */
            if (c == 7) ++r;
            else if (r == 0) ++c;
            else { --r; ++c; }
        } else { /* moving down-left */
            if (r == 7) ++c;
            else if (c == 0) ++r;
            else { ++r; --c; }
        }
    }
    g_init = 1;
}

void orc_zigzag(int32_t out[64]) {
    init_tables();
    for (int i = 0; i < 64; ++i) out[i] = g_zz[i];
}

/*
 * 8x8 inverse DCT by its definition (the inverse of the type-II transform of Section 2):
 *   f(y,x) = 1/4 * sum_u sum_v C(u) C(v) F(v,u) cos((2x+1) u pi/16) cos((2y+1) v pi/16)
 * F is row-major with v (vertical frequency) as the row.
 */
void orc_idct8x8(const double F[64], double f[64]) {
    init_tables();
    for (int y = 0; y < 8; ++y)
        for (int x = 0; x < 8; ++x) {
            double s = 0.0;
            for (int v = 0; v < 8; ++v)
                for (int u = 0; u < 8; ++u) s += F[v * 8 + u] * g_c[x][u] * g_c[y][v];
            f[y * 8 + x] = 0.25 * s;
        }
}

/* samples (double, level shift applied, not rounded) of data unit k: dequantise, undo zig-zag, IDCT, +128 */
static void unit_samples(const orc_image* im, const int16_t* coef, int64_t k, double out[64]) {
    int u = (int)(k % im->info.units_per_mcu);
    const uint16_t* q = im->info.qt[im->info.tq[im->unit_comp[u]]];
    double F[64];
    for (int i = 0; i < 64; ++i) F[g_zz[i]] = (double)coef[k * 64 + i] * (double)q[i];
    orc_idct8x8(F, out);
    for (int i = 0; i < 64; ++i) out[i] += 128.0;
}

static uint8_t to_u8(double v) {
    double r = floor(v + 0.5);
    if (r < 0) r = 0;
    if (r > 255) r = 255;
    return (uint8_t)r;
}

/*
 * Pixels of the rectangle of MCUs [mx0,mx1) x [my0,my1), written into the full-size
 * interleaved image `pixels` (height*width*ncomp bytes); parts outside the image are cropped.
 * Chroma is replicated to full resolution; YCbCr -> RGB with the JFIF matrix; the only
 * rounding is the final one.
 */
int orc_decode_pixels_mcus(const orc_image* im, const int16_t* coef, uint8_t* pixels, int mx0, int mx1, int my0,
                           int my1) {
    if (!im || !coef || !pixels) return ORC_E_ARG;
    init_tables();
    const orc_info* in = &im->info;
    if (mx0 < 0 || my0 < 0 || mx1 > in->mcus_x || my1 > in->mcus_y) return ORC_E_ARG;
    int mw = 8 * in->hmax, mh = 8 * in->vmax;
    double* plane = (double*)malloc(sizeof(double) * 3 * (size_t)mw * mh); /* one MCU, all components, full res */
    double blk[64];
    for (int my = my0; my < my1; ++my)
        for (int mx = mx0; mx < mx1; ++mx) {
            int64_t k0 = ((int64_t)my * in->mcus_x + mx) * in->units_per_mcu;
            for (int u = 0; u < in->units_per_mcu; ++u) {
                int c = im->unit_comp[u];
                unit_samples(im, coef, k0 + u, blk);
                int rx = in->hmax / in->hs[c], ry = in->vmax / in->vs[c]; /* replication factors */
                for (int y = 0; y < 8; ++y)
                    for (int x = 0; x < 8; ++x)
                        for (int dy = 0; dy < ry; ++dy)
                            for (int dx = 0; dx < rx; ++dx) {
                                int px = (im->unit_bx[u] * 8 + x) * rx + dx;
                                int py = (im->unit_by[u] * 8 + y) * ry + dy;
                                plane[((size_t)c * mh + py) * mw + px] = blk[y * 8 + x];
                            }
            }
            for (int y = 0; y < mh; ++y)
                for (int x = 0; x < mw; ++x) {
                    int gx = mx * mw + x, gy = my * mh + y;
                    if (gx >= in->width || gy >= in->height) continue;
                    uint8_t* o = pixels + ((size_t)gy * in->width + gx) * in->ncomp;
                    double Y = plane[((size_t)0 * mh + y) * mw + x];
                    if (in->ncomp == 1) { o[0] = to_u8(Y); continue; }
                    double Cb = plane[((size_t)1 * mh + y) * mw + x] - 128.0;
                    double Cr = plane[((size_t)2 * mh + y) * mw + x] - 128.0;
                    o[0] = to_u8(Y + 1.402 * Cr);
                    o[1] = to_u8(Y - 0.344136 * Cb - 0.714136 * Cr);
                    o[2] = to_u8(Y + 1.772 * Cb);
                }
        }
    free(plane);
    return ORC_OK;
}

int orc_decode_pixels(const orc_image* im, const int16_t* coef, uint8_t* pixels) {
    if (!im) return ORC_E_ARG;
    return orc_decode_pixels_mcus(im, coef, pixels, 0, im->info.mcus_x, 0, im->info.mcus_y);
}

/*
 * The decoder's output as the paper defines it (Section 3, problem statement: one array per colour channel;
 * Section 4.3: the inverse DCT is the last step when no upsampling or colour conversion is applied): the
 * samples of every component at the component's own resolution, level-shifted, rounded once and clamped.
 * Component c is plane_w[c] x plane_h[c] samples, ceil(width * hs[c] / hmax) by ceil(height * vs[c] / vmax)
 * (T.81 A.1.1); the planes are stored one after the other in `planes`.
 */
int orc_plane_size(const orc_image* im, int c, int32_t* w, int32_t* h) {
    if (!im || c < 0 || c >= im->info.ncomp) return ORC_E_ARG;
    const orc_info* in = &im->info;
    *w = (in->width * in->hs[c] + in->hmax - 1) / in->hmax;
    *h = (in->height * in->vs[c] + in->vmax - 1) / in->vmax;
    return ORC_OK;
}

int orc_decode_planes(const orc_image* im, const int16_t* coef, uint8_t* planes) {
    if (!im || !coef || !planes) return ORC_E_ARG;
    init_tables();
    const orc_info* in = &im->info;
    size_t base[3] = {0, 0, 0};
    int32_t pw[3], ph[3];
    size_t off = 0;
    for (int c = 0; c < in->ncomp; ++c) {
        orc_plane_size(im, c, &pw[c], &ph[c]);
        base[c] = off;
        off += (size_t)pw[c] * ph[c];
    }
    double blk[64];
    for (int my = 0; my < in->mcus_y; ++my)
        for (int mx = 0; mx < in->mcus_x; ++mx) {
            int64_t k0 = ((int64_t)my * in->mcus_x + mx) * in->units_per_mcu;
            for (int u = 0; u < in->units_per_mcu; ++u) {
                int c = im->unit_comp[u];
                unit_samples(im, coef, k0 + u, blk);
                for (int y = 0; y < 8; ++y)
                    for (int x = 0; x < 8; ++x) {
                        int gx = (mx * in->hs[c] + im->unit_bx[u]) * 8 + x;
                        int gy = (my * in->vs[c] + im->unit_by[u]) * 8 + y;
                        if (gx >= pw[c] || gy >= ph[c]) continue;
                        planes[base[c] + (size_t)gy * pw[c] + gx] = to_u8(blk[y * 8 + x]);
                    }
            }
        }
    return ORC_OK;
}

/* ------------------------------------------------------ reduced-size output */
/*
 * Output at 1/d of the size, d = 2, 4 or 8, computed in the transform domain (the paper stops at full-size
 * planes, Section 4.3, and names the inverse transform as the stage that now limits the decoder, Section 6;
 * a decoder that feeds a training pipeline usually wants a smaller image than the file holds and can skip
 * most of that stage).  The definition used here is the usual one for block transforms: of every data unit
 * only the n x n lowest frequencies are kept, n = 8 / d, and the n-point inverse transform of the same
 * family is applied to them,
 *   f(y,x) = 1/4 * sum_{u<n} sum_{v<n} C(u) C(v) F(v,u) cos((2x+1) u pi / (2n)) cos((2y+1) v pi / (2n)),
 * with the factor 1/4 of the 8-point transform kept, so that a unit that holds only a DC term keeps its
 * value (DC * Q / 8) at every size.  Every data unit thus yields n x n samples; everything after that is as
 * at full size: level shift, chroma replicated by the sampling factors, JFIF colour matrix, one rounding at
 * the very end, crop.  The output has ceil(width / d) x ceil(height / d) pixels; a component plane has
 * ceil(plane_w / d) x ceil(plane_h / d) samples.  d = 1 is the full-size path above.
 */
void orc_idct_scaled(const double F[64], int n, double* f) {
    const double pi = 3.14159265358979323846;
    for (int y = 0; y < n; ++y)
        for (int x = 0; x < n; ++x) {
            double s = 0.0;
            for (int v = 0; v < n; ++v)
                for (int u = 0; u < n; ++u) {
                    double cu = u == 0 ? 1.0 / sqrt(2.0) : 1.0, cv = v == 0 ? 1.0 / sqrt(2.0) : 1.0;
                    s += cu * cv * F[v * 8 + u] * cos((2 * x + 1) * u * pi / (2.0 * n)) * cos((2 * y + 1) * v * pi / (2.0 * n));
                }
            f[y * n + x] = 0.25 * s;
        }
}

static int scale_ok(int d) { return d == 1 || d == 2 || d == 4 || d == 8; }

/* n x n samples (double, level shift applied, not rounded) of data unit k at 1/d size, n = 8 / d */
static void unit_samples_scaled(const orc_image* im, const int16_t* coef, int64_t k, int n, double* out) {
    int u = (int)(k % im->info.units_per_mcu);
    const uint16_t* q = im->info.qt[im->info.tq[im->unit_comp[u]]];
    double F[64];
    for (int i = 0; i < 64; ++i) F[g_zz[i]] = (double)coef[k * 64 + i] * (double)q[i];
    orc_idct_scaled(F, n, out);
    for (int i = 0; i < n * n; ++i) out[i] += 128.0;
}

int orc_scaled_size(const orc_image* im, int d, int32_t* w, int32_t* h) {
    if (!im || !scale_ok(d)) return ORC_E_ARG;
    *w = (im->info.width + d - 1) / d;
    *h = (im->info.height + d - 1) / d;
    return ORC_OK;
}

int orc_scaled_plane_size(const orc_image* im, int d, int c, int32_t* w, int32_t* h) {
    if (!im || !scale_ok(d)) return ORC_E_ARG;
    int32_t pw, ph;
    int rc = orc_plane_size(im, c, &pw, &ph);
    if (rc) return rc;
    *w = (pw + d - 1) / d;
    *h = (ph + d - 1) / d;
    return ORC_OK;
}

/* interleaved gray or RGB image of ceil(height/d) x ceil(width/d) pixels */
int orc_decode_pixels_scaled(const orc_image* im, const int16_t* coef, int d, uint8_t* pixels) {
    if (!im || !coef || !pixels || !scale_ok(d)) return ORC_E_ARG;
    init_tables();
    const orc_info* in = &im->info;
    const int n = 8 / d;
    int32_t ow, oh;
    orc_scaled_size(im, d, &ow, &oh);
    int mw = n * in->hmax, mh = n * in->vmax; /* output pixels per MCU */
    double* plane = (double*)malloc(sizeof(double) * 3 * (size_t)mw * mh);
    double blk[64];
    for (int my = 0; my < in->mcus_y; ++my)
        for (int mx = 0; mx < in->mcus_x; ++mx) {
            int64_t k0 = ((int64_t)my * in->mcus_x + mx) * in->units_per_mcu;
            for (int u = 0; u < in->units_per_mcu; ++u) {
                int c = im->unit_comp[u];
                unit_samples_scaled(im, coef, k0 + u, n, blk);
                int rx = in->hmax / in->hs[c], ry = in->vmax / in->vs[c];
                for (int y = 0; y < n; ++y)
                    for (int x = 0; x < n; ++x)
                        for (int dy = 0; dy < ry; ++dy)
                            for (int dx = 0; dx < rx; ++dx) {
                                int px = (im->unit_bx[u] * n + x) * rx + dx;
                                int py = (im->unit_by[u] * n + y) * ry + dy;
                                plane[((size_t)c * mh + py) * mw + px] = blk[y * n + x];
                            }
            }
            for (int y = 0; y < mh; ++y)
                for (int x = 0; x < mw; ++x) {
                    int gx = mx * mw + x, gy = my * mh + y;
                    if (gx >= ow || gy >= oh) continue;
                    uint8_t* o = pixels + ((size_t)gy * ow + gx) * in->ncomp;
                    double Y = plane[((size_t)0 * mh + y) * mw + x];
                    if (in->ncomp == 1) { o[0] = to_u8(Y); continue; }
                    double Cb = plane[((size_t)1 * mh + y) * mw + x] - 128.0;
                    double Cr = plane[((size_t)2 * mh + y) * mw + x] - 128.0;
                    o[0] = to_u8(Y + 1.402 * Cr);
                    o[1] = to_u8(Y - 0.344136 * Cb - 0.714136 * Cr);
                    o[2] = to_u8(Y + 1.772 * Cb);
                }
        }
    free(plane);
    return ORC_OK;
}

/* the component planes at 1/d size, one after the other */
int orc_decode_planes_scaled(const orc_image* im, const int16_t* coef, int d, uint8_t* planes) {
    if (!im || !coef || !planes || !scale_ok(d)) return ORC_E_ARG;
    init_tables();
    const orc_info* in = &im->info;
    const int n = 8 / d;
    size_t base[3] = {0, 0, 0};
    int32_t pw[3], ph[3];
    size_t off = 0;
    for (int c = 0; c < in->ncomp; ++c) {
        orc_scaled_plane_size(im, d, c, &pw[c], &ph[c]);
        base[c] = off;
        off += (size_t)pw[c] * ph[c];
    }
    double blk[64];
    for (int my = 0; my < in->mcus_y; ++my)
        for (int mx = 0; mx < in->mcus_x; ++mx) {
            int64_t k0 = ((int64_t)my * in->mcus_x + mx) * in->units_per_mcu;
            for (int u = 0; u < in->units_per_mcu; ++u) {
                int c = im->unit_comp[u];
                unit_samples_scaled(im, coef, k0 + u, n, blk);
                for (int y = 0; y < n; ++y)
                    for (int x = 0; x < n; ++x) {
                        int gx = (mx * in->hs[c] + im->unit_bx[u]) * n + x;
                        int gy = (my * in->vs[c] + im->unit_by[u]) * n + y;
                        if (gx >= pw[c] || gy >= ph[c]) continue;
                        planes[base[c] + (size_t)gy * pw[c] + gx] = to_u8(blk[y * n + x]);
                    }
            }
        }
    return ORC_OK;
}
