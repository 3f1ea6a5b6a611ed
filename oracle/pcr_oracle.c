/*
 * pcr_oracle -- plain, slow CPU reference for decoding Progressive Compressed Records.
 *
 * TEST INFRASTRUCTURE ONLY.  This file exists to say what the GPU library must compute; it
 * is called from tests, from the smoke check and from the benchmark's CPU-baseline leg, and
 * from nowhere else.  It shares no code, table or header with the GPU library.
 *
 * What it follows:
 *   - the record layout, the prefix rule ("read from the start of the record to the end of
 *     scan group k") and the re-serialisation of each image's scans followed by an
 *     end-of-image marker: paper Section 3 (record figure) and Section 5 ("Encoding", "Decoding");
 *   - what the bytes of one image mean: the JPEG standard (ITU-T T.81) -- marker syntax
 *     (Annex B), Huffman table construction (Annex C), sequential Huffman decoding (F.2.2),
 *     progressive decoding with spectral selection and successive approximation (Annex G),
 *     the inverse DCT (A.3.3) -- and the JFIF colour convention.  The paper delegates this
 *     step to a stock decoder (Section 5, "Decoding"; Section 4.2).
 * Where the standard leaves a choice (what to show for coefficients not yet received,
 * chroma up-sampling, rounding) the choices are: missing coefficients are zero and no
 * smoothing is applied; chroma samples are replicated; samples stay in floating point
 * (clamped to [0,255] per component) until one final round-half-up.  A triangle-filter
 * up-sampler with per-component rounding is provided only to compare against stock decoders.
 *
 * Pins: every function below is pinned by tests that do not rely on this file alone
 * (byte identity of reassembly, encoder round trips on random coefficients, sequential-vs-
 * progressive equality, streams made by an independent encoder and compared with an
 * independent decoder, the O(N^4) DCT definition, closed forms).  One part is NOT pinned
 * by anything but this file: the *pixels* of a truncated stream (k < number of scans)
 * beyond structural properties -- parity unpinned for that case.
 *
 * Plain C99; doubles throughout the pixel stage.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_OK = 0, ORC_E_ARG = -1, ORC_E_FORMAT = -2, ORC_E_TRUNCATED = -3, ORC_E_UNSUPPORTED = -4, ORC_E_RANGE = -5 };

/* =========================================================================================
 * Part A.  Record level (paper Section 3).
 * ======================================================================================= */
static uint32_t rd32(const uint8_t* p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24); }
static uint64_t rd64(const uint8_t* p) { return (uint64_t)rd32(p) | ((uint64_t)rd32(p + 4) << 32); }

/* Header fields; returns ORC_OK and the number of scan groups wholly contained in nbytes. */
int orc_record_header(const uint8_t* rec, size_t nbytes, uint32_t* n, uint32_t* G, uint64_t* header_bytes, int* k_avail) {
    if (!rec || nbytes < 24) return ORC_E_TRUNCATED;
    if (memcmp(rec, "PCR1", 4) != 0) return ORC_E_FORMAT;
    uint32_t version = rd32(rec + 4);
    if (version != 1 && version != 2) return ORC_E_UNSUPPORTED;
    *n = rd32(rec + 8); *G = rd32(rec + 12); *header_bytes = rd64(rec + 16);
    if (*n == 0 || *G == 0) return ORC_E_FORMAT;
    uint64_t need = 24 + 8ull * *G + 8ull * *n + 4ull * *G * *n;
    if (version == 2) need += 8 + 2ull * *G * *n;            /* entry interval, reserved word, entry counts */
    if (*header_bytes < need) return ORC_E_FORMAT;
    if (nbytes < *header_bytes) return ORC_E_TRUNCATED;
    int k = 0; uint64_t prev = *header_bytes;
    for (uint32_t g = 0; g < *G; g++) {
        uint64_t e = rd64(rec + 24 + 8 * g);
        if (e < prev) return ORC_E_FORMAT;
        if (e <= nbytes && k == (int)g) k = (int)g + 1;
        prev = e;
    }
    *k_avail = k;
    return ORC_OK;
}

/* The ungrouping index: off[g*n+i] = absolute offset of image i's region in group g+1, i.e.
 * the start of the group plus the lengths of the images before it; len likewise. */
int orc_record_index(const uint8_t* rec, size_t nbytes, uint64_t* off, uint32_t* len, int32_t* label, uint32_t* nscans, uint64_t* group_end) {
    uint32_t n, G; uint64_t hb; int k;
    int rc = orc_record_header(rec, nbytes, &n, &G, &hb, &k);
    if (rc) return rc;
    const uint8_t* p = rec + 24;
    for (uint32_t g = 0; g < G; g++) if (group_end) group_end[g] = rd64(p + 8 * g);
    const uint8_t* pl = p + 8 * (size_t)G;
    const uint8_t* pn = pl + 4 * (size_t)n;
    const uint8_t* pz = pn + 4 * (size_t)n;
    for (uint32_t i = 0; i < n; i++) { if (label) label[i] = (int32_t)rd32(pl + 4 * i); if (nscans) nscans[i] = rd32(pn + 4 * i); }
    /* Version 2 records end every group with decoder hints (places inside the scans where a decoder may start),
     * as many per image as the count table behind the length table says: the low 15 bits of an entry of that
     * table are the count, the top bit says that the hints of this scan are 8 bytes each instead of 16.  A plain
     * decoder has no use for them: they are skipped, and only their size enters the check that the group is tiled. */
    const uint8_t* pe = rd32(rec + 4) == 2 ? pz + 4 * (size_t)G * n + 8 : NULL;
    uint64_t start = hb;
    for (uint32_t g = 0; g < G; g++) {
        uint64_t pos = start;
        for (uint32_t i = 0; i < n; i++) {
            uint32_t L = rd32(pz + 4 * ((size_t)g * n + i));
            off[(size_t)g * n + i] = pos; len[(size_t)g * n + i] = L; pos += L;
        }
        if (pe) for (uint32_t i = 0; i < n; i++) {
            const uint8_t* c = pe + 2 * ((size_t)g * n + i);
            const uint32_t field = c[0] | ((uint32_t)c[1] << 8);
            pos += (uint64_t)(field & 0x7FFFu) * ((field & 0x8000u) ? 8u : 16u);
        }
        if (pos != rd64(p + 8 * g)) return ORC_E_FORMAT;      /* regions (and hints) must tile the group */
        start = pos;
    }
    return ORC_OK;
}

/* Byte string handed to the image decoder for image i at fidelity k: regions 1..min(k, scans
 * of i) in order, then FF D9 if and only if scans were left out.  Returns its length through
 * *out_len (dst may be NULL to query). */
int orc_reassemble(const uint8_t* rec, size_t nbytes, uint32_t i, int k, uint8_t* dst, size_t cap, size_t* out_len) {
    uint32_t n, G; uint64_t hb; int kav;
    int rc = orc_record_header(rec, nbytes, &n, &G, &hb, &kav);
    if (rc) return rc;
    if (i >= n || k < 1 || k > (int)G) return ORC_E_RANGE;
    if (k > kav) return ORC_E_TRUNCATED;
    uint64_t* off = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)G * n);
    uint32_t* len = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)G * n);
    uint32_t* ns = (uint32_t*)malloc(sizeof(uint32_t) * n);
    rc = orc_record_index(rec, nbytes, off, len, NULL, ns, NULL);
    size_t w = 0;
    if (!rc) {
        int have = k < (int)ns[i] ? k : (int)ns[i];
        for (int g = 0; g < have; g++) {
            size_t L = len[(size_t)g * n + i];
            if (dst) { if (w + L > cap) { rc = ORC_E_RANGE; break; } memcpy(dst + w, rec + off[(size_t)g * n + i], L); }
            w += L;
        }
        if (!rc && have < (int)ns[i]) {
            if (dst) { if (w + 2 > cap) rc = ORC_E_RANGE; else { dst[w] = 0xFF; dst[w + 1] = 0xD9; } }
            w += 2;
        }
    }
    free(off); free(len); free(ns);
    if (!rc) *out_len = w;
    return rc;
}

/* =========================================================================================
 * Part B.  One image: markers and entropy decoding (T.81 Annexes B, C, F.2.2, G).
 * ======================================================================================= */
typedef struct {
    int defined;
    int mincode[17], maxcode[17], valptr[17];   /* per code length */
    uint8_t huffval[256];
} htab_t;

typedef struct {
    int W, H, nc, progressive;
    int cid[3], hs[3], vs[3], tq[3];
    int hmax, vmax, mcux, mcuy;
    int bw[3], bh[3];          /* allocated block grid (MCU padded) */
    int cw[3], ch[3];          /* blocks that cover the component's own samples */
    uint16_t q[4][64];         /* zig-zag order as stored */
    int qdef[4];
    htab_t dc[4], ac[4];
    int ri;
    int16_t* coef[3];
    int zz[64];
    int nscan_c[3], dc_first_c[3];   /* per component: scans received that carry it; DC first scans among them */
} dec_t;

static void gen_zigzag(int zz[64]) {
    /* walk the anti-diagonals u+v = s, alternating direction, first move to the right */
    int v = 0, u = 0;
    for (int i = 0; i < 64; i++) {
        zz[i] = v * 8 + u;
        if (((u + v) & 1) == 0) {           /* moving up-right */
            if (u == 7) v++; else if (v == 0) u++; else { u++; v--; }
        } else {                             /* moving down-left */
            if (v == 7) u++; else if (u == 0) v++; else { u--; v++; }
        }
    }
}

static void build_htab(htab_t* t, const uint8_t bits[16], const uint8_t* vals, int nvals) {
    memset(t, 0, sizeof *t);
    t->defined = 1;
    memcpy(t->huffval, vals, (size_t)nvals);
    int code = 0, k = 0;
    for (int l = 1; l <= 16; l++) {
        if (bits[l - 1]) {
            t->valptr[l] = k; t->mincode[l] = code;
            code += bits[l - 1]; k += bits[l - 1];
            t->maxcode[l] = code - 1;
        } else t->maxcode[l] = -1;
        code <<= 1;
    }
}

/* bit reader over one entropy-coded segment [p, end): removes stuffed zeros, stops at markers */
typedef struct { const uint8_t* p; const uint8_t* end; int bitpos; int err; } bits_t;

static int next_bit(bits_t* b) {
    if (b->err) return 0;
    if (b->p >= b->end) { b->err = 1; return 0; }
    if (b->bitpos == 0 && b->p[0] == 0xFF) {
        /* FF must be followed by 00 to be data */
        if (b->p + 1 >= b->end || b->p[1] != 0x00) { b->err = 1; return 0; }
    }
    int bit = (b->p[0] >> (7 - b->bitpos)) & 1;
    if (++b->bitpos == 8) { b->bitpos = 0; b->p += (b->p[0] == 0xFF) ? 2 : 1; }
    return bit;
}
static int receive(bits_t* b, int n) { int v = 0; while (n--) v = (v << 1) | next_bit(b); return v; }
static int extend(int v, int s) { return (s && v < (1 << (s - 1))) ? v - (1 << s) + 1 : v; }
static int huff_decode(bits_t* b, const htab_t* t) {
    int code = 0;
    for (int l = 1; l <= 16; l++) {
        code = (code << 1) | next_bit(b);
        if (b->err) return 0;
        if (t->maxcode[l] >= 0 && code <= t->maxcode[l] && code >= t->mincode[l]) return t->huffval[t->valptr[l] + code - t->mincode[l]];
    }
    b->err = 1;
    return 0;
}
/* at a restart boundary: drop the rest of the current byte, expect FF Dm */
static void take_restart(bits_t* b, int m) {
    if (b->err) return;
    if (b->bitpos) { b->p += (b->p[0] == 0xFF) ? 2 : 1; b->bitpos = 0; }
    while (b->p + 2 < b->end && b->p[0] == 0xFF && b->p[1] == 0xFF) b->p++;    /* fill bytes */
    if (b->p + 2 > b->end || b->p[0] != 0xFF || b->p[1] != 0xD0 + (m & 7)) { b->err = 1; return; }
    b->p += 2;
}

typedef struct { int ns, c[3], td[3], ta[3], Ss, Se, Ah, Al; } scanhdr_t;

static void dc_first(dec_t* D, bits_t* b, int c, int td, int Al, int16_t* blk, int* pred) {
    int t = huff_decode(b, &D->dc[td]);
    if (t > 15) { b->err = 1; return; }
    int diff = t ? extend(receive(b, t), t) : 0;
    pred[c] += diff;
    if (!b->err) blk[0] = (int16_t)(pred[c] * (1 << Al));
}

static void ac_first(dec_t* D, bits_t* b, int ta, int Ss, int Se, int Al, int16_t* blk, int* eobrun) {
    if (*eobrun > 0) { (*eobrun)--; return; }
    int k = Ss;
    while (k <= Se) {
        int rs = huff_decode(b, &D->ac[ta]);
        if (b->err) return;
        int r = rs >> 4, s = rs & 15;
        if (s) {
            k += r;
            if (k > Se) { b->err = 1; return; }
            int v = extend(receive(b, s), s);
            if (b->err) return;
            blk[D->zz[k]] = (int16_t)(v * (1 << Al));
            k++;
        } else if (r == 15) k += 16;
        else { *eobrun = (1 << r) - 1 + (r ? receive(b, r) : 0); return; }
    }
}

static void correct(bits_t* b, int16_t* c, int p) {
    if (next_bit(b) && !b->err) *c = (int16_t)(*c > 0 ? *c + p : *c - p);   /* magnitude grows by p */
}

static void ac_refine(dec_t* D, bits_t* b, int ta, int Ss, int Se, int Al, int16_t* blk, int* eobrun) {
    int p = 1 << Al, k = Ss;
    if (*eobrun == 0) {
        while (k <= Se) {
            int rs = huff_decode(b, &D->ac[ta]);
            if (b->err) return;
            int r = rs >> 4, s = rs & 15, newval = 0;
            if (s == 1) newval = next_bit(b) ? p : -p;
            else if (s != 0) { b->err = 1; return; }
            else if (r < 15) { *eobrun = (1 << r) + (r ? receive(b, r) : 0); break; }
            /* pass over coefficients: corrections for the non-zero ones, count down r on zeros */
            while (k <= Se) {
                int16_t* c = &blk[D->zz[k]];
                if (*c != 0) correct(b, c, p);
                else { if (r == 0) { if (newval) *c = (int16_t)newval; break; } r--; }
                if (b->err) return;
                k++;
            }
            if (newval && k > Se) { b->err = 1; return; }   /* ran off the band before placing it */
            k++;
        }
    }
    if (*eobrun > 0) {
        for (; k <= Se; k++) { int16_t* c = &blk[D->zz[k]]; if (*c != 0) correct(b, c, p); if (b->err) return; }
        (*eobrun)--;
    }
}

/* sequential (non-progressive) block: DC difference then AC run/size pairs, 00 = end of block */
static void seq_block(dec_t* D, bits_t* b, int c, int td, int ta, int16_t* blk, int* pred) {
    dc_first(D, b, c, td, 0, blk, pred);
    int k = 1;
    while (k < 64 && !b->err) {
        int rs = huff_decode(b, &D->ac[ta]);
        int r = rs >> 4, s = rs & 15;
        if (s) { k += r; if (k > 63) { b->err = 1; return; } blk[D->zz[k]] = (int16_t)extend(receive(b, s), s); k++; }
        else if (r == 15) k += 16;
        else break;
    }
}

static int decode_scan(dec_t* D, const scanhdr_t* S, const uint8_t* seg, const uint8_t* seg_end) {
    bits_t b = { seg, seg_end, 0, 0 };
    int pred[3] = {0, 0, 0}, eobrun = 0;
    long mcu_w, mcu_n;
    if (S->ns > 1) { mcu_w = D->mcux; mcu_n = (long)D->mcux * D->mcuy; }
    else { mcu_w = D->cw[S->c[0]]; mcu_n = (long)D->cw[S->c[0]] * D->ch[S->c[0]]; }
    int rst = 0;
    for (long m = 0; m < mcu_n; m++) {
        if (D->ri > 0 && m > 0 && m % D->ri == 0) {
            take_restart(&b, rst); rst++;
            pred[0] = pred[1] = pred[2] = 0; eobrun = 0;
        }
        long my = m / mcu_w, mx = m % mcu_w;
        for (int j = 0; j < S->ns; j++) {
            int c = S->c[j];
            int nx = S->ns > 1 ? D->hs[c] : 1, ny = S->ns > 1 ? D->vs[c] : 1;
            for (int by = 0; by < ny; by++) for (int bx = 0; bx < nx; bx++) {
                long row = S->ns > 1 ? my * D->vs[c] + by : my, col = S->ns > 1 ? mx * D->hs[c] + bx : mx;
                int16_t* blk = D->coef[c] + ((size_t)row * D->bw[c] + col) * 64;
                if (!D->progressive) seq_block(D, &b, c, S->td[j], S->ta[j], blk, pred);
                else if (S->Ss == 0) {
                    if (S->Ah == 0) dc_first(D, &b, c, S->td[j], S->Al, blk, pred);
                    else if (next_bit(&b)) blk[0] |= (int16_t)(1 << S->Al);
                } else if (S->Ah == 0) ac_first(D, &b, S->ta[j], S->Ss, S->Se, S->Al, blk, &eobrun);
                else ac_refine(D, &b, S->ta[j], S->Ss, S->Se, S->Al, blk, &eobrun);
                if (b.err) return ORC_E_FORMAT;
            }
        }
    }
    return ORC_OK;
}

typedef struct { int W, H, nc, hs[3], vs[3], bw[3], bh[3], nscans, progressive; } orc_info_t;

static void setup_geometry(dec_t* D) {
    D->hmax = D->vmax = 1;
    for (int c = 0; c < D->nc; c++) { if (D->hs[c] > D->hmax) D->hmax = D->hs[c]; if (D->vs[c] > D->vmax) D->vmax = D->vs[c]; }
    D->mcux = (D->W + 8 * D->hmax - 1) / (8 * D->hmax); D->mcuy = (D->H + 8 * D->vmax - 1) / (8 * D->vmax);
    for (int c = 0; c < D->nc; c++) {
        D->bw[c] = D->mcux * D->hs[c]; D->bh[c] = D->mcuy * D->vs[c];
        int xc = (D->W * D->hs[c] + D->hmax - 1) / D->hmax, yc = (D->H * D->vs[c] + D->vmax - 1) / D->vmax;
        D->cw[c] = (xc + 7) / 8; D->ch[c] = (yc + 7) / 8;
    }
}

/* Walk the markers of one JPEG byte string.  With coef == NULL only the frame header is
 * read (info filled in).  Otherwise every scan found is decoded into coef (planes
 * concatenated, [bh][bw][64], natural order, zero initialised here). */
static int walk(const uint8_t* d, size_t n, dec_t* D, orc_info_t* info, int16_t* coef) {
    if (n < 4 || d[0] != 0xFF || d[1] != 0xD8) return ORC_E_FORMAT;
    size_t p = 2; int have_frame = 0, nscans = 0;
    memset(D, 0, sizeof *D); gen_zigzag(D->zz);
    while (1) {
        if (p + 2 > n) return ORC_E_FORMAT;               /* ran out before EOI */
        if (d[p] != 0xFF) return ORC_E_FORMAT;
        int m = d[p + 1];
        if (m == 0xFF) { p++; continue; }
        if (m == 0xD9) break;
        if (p + 4 > n) return ORC_E_FORMAT;
        size_t L = ((size_t)d[p + 2] << 8) | d[p + 3];
        if (L < 2 || p + 2 + L > n) return ORC_E_FORMAT;
        const uint8_t* s = d + p + 4; const uint8_t* se = d + p + 2 + L;
        p += 2 + L;
        if (m == 0xDB) {
            while (s < se) {
                int pq = s[0] >> 4, tq = s[0] & 15; s++;
                if (tq > 3 || pq > 1) return ORC_E_FORMAT;
                if (s + 64 * (pq + 1) > se) return ORC_E_FORMAT;
                for (int i = 0; i < 64; i++) { D->q[tq][i] = pq ? (uint16_t)((s[0] << 8) | s[1]) : s[0]; s += pq + 1; }
                D->qdef[tq] = 1;
            }
        } else if (m == 0xC0 || m == 0xC1 || m == 0xC2) {
            if (have_frame) return ORC_E_FORMAT;
            if (se - s < 6) return ORC_E_FORMAT;
            if (s[0] != 8) return ORC_E_UNSUPPORTED;
            D->progressive = (m == 0xC2);
            D->H = (s[1] << 8) | s[2]; D->W = (s[3] << 8) | s[4]; D->nc = s[5];
            if (D->H == 0 || D->W == 0) return ORC_E_UNSUPPORTED;
            if (D->nc != 1 && D->nc != 3) return ORC_E_UNSUPPORTED;
            if (se - s < 6 + 3 * D->nc) return ORC_E_FORMAT;
            for (int c = 0; c < D->nc; c++) {
                D->cid[c] = s[6 + 3 * c]; D->hs[c] = s[7 + 3 * c] >> 4; D->vs[c] = s[7 + 3 * c] & 15; D->tq[c] = s[8 + 3 * c];
                if (D->hs[c] < 1 || D->hs[c] > 2 || D->vs[c] < 1 || D->vs[c] > 2 || D->tq[c] > 3) return ORC_E_UNSUPPORTED;
            }
            if (D->nc == 1) D->hs[0] = D->vs[0] = 1;      /* a single component is never subsampled */
            setup_geometry(D);
            have_frame = 1;
            info->W = D->W; info->H = D->H; info->nc = D->nc; info->progressive = D->progressive;
            size_t o = 0;
            for (int c = 0; c < D->nc; c++) {
                info->hs[c] = D->hs[c]; info->vs[c] = D->vs[c]; info->bw[c] = D->bw[c]; info->bh[c] = D->bh[c];
                if (coef) D->coef[c] = coef + o;
                o += (size_t)D->bw[c] * D->bh[c] * 64;
            }
            if (coef) memset(coef, 0, o * sizeof(int16_t));
        } else if (m >= 0xC3 && m <= 0xCF && m != 0xC4 && m != 0xC8 && m != 0xCC) {
            return ORC_E_UNSUPPORTED;                      /* lossless, hierarchical, arithmetic */
        } else if (m == 0xC4) {
            while (s < se) {
                int tc = s[0] >> 4, th = s[0] & 15;
                if (tc > 1 || th > 3 || s + 17 > se) return ORC_E_FORMAT;
                int nv = 0; for (int i = 0; i < 16; i++) nv += s[1 + i];
                if (nv > 256 || s + 17 + nv > se) return ORC_E_FORMAT;
                build_htab(tc ? &D->ac[th] : &D->dc[th], s + 1, s + 17, nv);
                s += 17 + nv;
            }
        } else if (m == 0xDD) {
            if (se - s < 2) return ORC_E_FORMAT;
            D->ri = (s[0] << 8) | s[1];
        } else if (m == 0xDC) {
            return ORC_E_UNSUPPORTED;                      /* DNL */
        } else if (m == 0xDA) {
            if (!have_frame) return ORC_E_FORMAT;
            scanhdr_t S; memset(&S, 0, sizeof S);
            if (se - s < 1) return ORC_E_FORMAT;
            S.ns = s[0];
            if (S.ns < 1 || S.ns > D->nc || se - s < 1 + 2 * S.ns + 3) return ORC_E_FORMAT;
            for (int j = 0; j < S.ns; j++) {
                int id = s[1 + 2 * j], c = -1;
                for (int q = 0; q < D->nc; q++) if (D->cid[q] == id) c = q;
                if (c < 0) return ORC_E_FORMAT;
                S.c[j] = c; S.td[j] = s[2 + 2 * j] >> 4; S.ta[j] = s[2 + 2 * j] & 15;
                if (S.td[j] > 3 || S.ta[j] > 3) return ORC_E_FORMAT;
            }
            S.Ss = s[1 + 2 * S.ns]; S.Se = s[2 + 2 * S.ns]; S.Ah = s[3 + 2 * S.ns] >> 4; S.Al = s[3 + 2 * S.ns] & 15;
            if (D->progressive) {
                if (S.Ss > S.Se || S.Se > 63 || (S.Ss == 0 && S.Se != 0) || (S.Ss > 0 && S.ns != 1) || S.Al > 13) return ORC_E_FORMAT;
            } else if (S.Ss != 0 || S.Se != 63 || S.Ah != 0 || S.Al != 0) return ORC_E_FORMAT;
            /* entropy-coded segment: up to the next marker that is not RSTm / stuffed zero */
            size_t e = p;
            while (1) {
                while (e < n && d[e] != 0xFF) e++;
                if (e + 1 >= n) return ORC_E_FORMAT;
                int x = d[e + 1];
                if (x == 0x00 || (x >= 0xD0 && x <= 0xD7)) { e += 2; continue; }
                if (x == 0xFF) { e++; continue; }
                break;
            }
            nscans++;
            for (int j = 0; j < S.ns; j++) { D->nscan_c[S.c[j]]++; if (D->progressive && S.Ss == 0 && S.Se == 0 && S.Ah == 0) D->dc_first_c[S.c[j]]++; }
            if (coef) {
                for (int j = 0; j < S.ns; j++) {
                    int needs_dc = !D->progressive || (S.Ss == 0 && S.Ah == 0), needs_ac = !D->progressive || S.Ss > 0;
                    if (needs_dc && !D->dc[S.td[j]].defined) return ORC_E_FORMAT;
                    if (needs_ac && !D->ac[S.ta[j]].defined) return ORC_E_FORMAT;
                }
                int rc = decode_scan(D, &S, d + p, d + e);
                if (rc) return rc;
            }
            p = e;
        }
        /* APPn, COM and anything else with a length: skipped */
    }
    if (!have_frame) return ORC_E_FORMAT;
    info->nscans = nscans;
    return ORC_OK;
}

int orc_image_info(const uint8_t* jpg, size_t n, orc_info_t* info) {
    dec_t* D = (dec_t*)malloc(sizeof(dec_t));
    int rc = walk(jpg, n, D, info, NULL);
    free(D);
    return rc;
}

/* =========================================================================================
 * Part C.  Pixels: dequantise, inverse DCT, up-sample, colour (T.81 A.3.3; JFIF).
 * ======================================================================================= */
#define PI 3.14159265358979323846

/* the definition, evaluated term by term: f(y,x) = 1/4 sum_u sum_v C(u)C(v) F(v,u) cos.. cos.. */
void orc_idct_direct(const double F[64], double f[64]) {
    for (int y = 0; y < 8; y++) for (int x = 0; x < 8; x++) {
        double a = 0;
        for (int v = 0; v < 8; v++) for (int u = 0; u < 8; u++) {
            double cu = u ? 1.0 : sqrt(0.5), cv = v ? 1.0 : sqrt(0.5);
            a += cu * cv * F[v * 8 + u] * cos((2 * x + 1) * u * PI / 16) * cos((2 * y + 1) * v * PI / 16);
        }
        f[y * 8 + x] = a / 4;
    }
}
/* same sum, rows then columns */
void orc_idct_separable(const double F[64], double f[64]) {
    double b[8][8], t[64];
    for (int u = 0; u < 8; u++) for (int x = 0; x < 8; x++) b[u][x] = (u ? 1.0 : sqrt(0.5)) * cos((2 * x + 1) * u * PI / 16) / 2;
    for (int v = 0; v < 8; v++) for (int x = 0; x < 8; x++) { double a = 0; for (int u = 0; u < 8; u++) a += F[v * 8 + u] * b[u][x]; t[v * 8 + x] = a; }
    for (int y = 0; y < 8; y++) for (int x = 0; x < 8; x++) { double a = 0; for (int v = 0; v < 8; v++) a += t[v * 8 + x] * b[v][y]; f[y * 8 + x] = a; }
}

static double clamp255(double v) { return v < 0 ? 0 : (v > 255 ? 255 : v); }

/* coefficient planes -> component sample planes (doubles, clamped to [0,255], not rounded) */
static void planes_from_coefs(const dec_t* D, int idct_direct, double* plane[3]) {
    for (int c = 0; c < D->nc; c++) {
        int pw = D->bw[c] * 8;
        const uint16_t* q = D->q[D->tq[c]];
        for (int by = 0; by < D->bh[c]; by++) for (int bx = 0; bx < D->bw[c]; bx++) {
            const int16_t* blk = D->coef[c] + ((size_t)by * D->bw[c] + bx) * 64;
            double F[64], f[64];
            for (int k = 0; k < 64; k++) F[D->zz[k]] = (double)blk[D->zz[k]] * q[k];
            if (idct_direct) orc_idct_direct(F, f); else orc_idct_separable(F, f);
            for (int y = 0; y < 8; y++) for (int x = 0; x < 8; x++)
                plane[c][(size_t)(by * 8 + y) * pw + bx * 8 + x] = clamp255(f[y * 8 + x] + 128.0);
        }
    }
}

static uint8_t round_u8(double v) { v = floor(v + 0.5); return (uint8_t)(v < 0 ? 0 : (v > 255 ? 255 : v)); }

/* triangle filter along one axis on a rounded plane, for comparison with stock decoders only:
 * each output is 3/4 of the nearer input sample plus 1/4 of the farther one */
static double tri(const double* p, int n, int stride, int i2) {
    int i = i2 >> 1, j = (i2 & 1) ? i + 1 : i - 1;
    if (j < 0) j = 0;
    if (j >= n) j = n - 1;
    return 0.75 * p[(size_t)i * stride] + 0.25 * p[(size_t)j * stride];
}

/*
 * Smoothing of a component of which only the DC first scan has been received (T.81 K.8: the five lowest AC
 * coefficients of a block are predicted from the DC coefficients of the block and its eight neighbours, the
 * coefficients of the quadratic surface whose means over the nine blocks are the nine DC values).  In the integer
 * form used here the weights are 36/256, 9/256 and 5/256 of the de-quantised DC differences, and the prediction is
 * rounded to a multiple of the coefficient's own quantiser step, halves away from zero:
 *     zig-zag 1 (horizontal frequency 1):  36 (left - right)
 *     zig-zag 2 (vertical frequency 1):    36 (above - below)
 *     zig-zag 3 (vertical frequency 2):     9 (above + below - 2 centre)
 *     zig-zag 4 (one of each):              5 ((above-left - above-right) - (below-left - below-right))
 *     zig-zag 5 (horizontal frequency 2):   9 (left + right - 2 centre)
 * A neighbour beyond the component's block grid is the nearest block inside it.  Predictions are limited to
 * +-1023, the range of an AC coefficient of 8-bit samples.  Components that have received anything besides
 * their DC first scan, and sequential files, are left as they are.
 */
static int16_t predict(int64_t w, int64_t q0, int64_t delta, int64_t qz) {
    if (qz == 0) return 0;   /* (a step the standard does not allow: the coefficient would de-quantise to zero anyway) */
    int64_t num = w * q0 * delta, den = 256 * qz, v = num >= 0 ? (num + den / 2) / den : -((-num + den / 2) / den);
    if (v > 1023) v = 1023;
    if (v < -1023) v = -1023;
    return (int16_t)v;
}
static void smooth_dc_only_components(dec_t* D) {
    for (int c = 0; c < D->nc; c++) {
        if (!D->progressive || D->nscan_c[c] != 1 || D->dc_first_c[c] != 1) continue;
        const uint16_t* q = D->q[D->tq[c]];
        int bw = D->bw[c], bh = D->bh[c];
        for (int by = 0; by < bh; by++) for (int bx = 0; bx < bw; bx++) {
            int64_t d[3][3];
            for (int dy = -1; dy <= 1; dy++) for (int dx = -1; dx <= 1; dx++) {
                int y = by + dy, x = bx + dx;
                y = y < 0 ? 0 : (y >= bh ? bh - 1 : y); x = x < 0 ? 0 : (x >= bw ? bw - 1 : x);
                d[dy + 1][dx + 1] = D->coef[c][((size_t)y * bw + x) * 64];
            }
            int16_t* blk = D->coef[c] + ((size_t)by * bw + bx) * 64;
            /* (blk is in natural order: index 8 v + u; q in zig-zag order) */
            blk[1]  = predict(36, q[0], d[1][0] - d[1][2], q[1]);
            blk[8]  = predict(36, q[0], d[0][1] - d[2][1], q[2]);
            blk[16] = predict(9,  q[0], d[0][1] + d[2][1] - 2 * d[1][1], q[3]);
            blk[9]  = predict(5,  q[0], (d[0][0] - d[0][2]) - (d[2][0] - d[2][2]), q[4]);
            blk[2]  = predict(9,  q[0], d[1][0] + d[1][2] - 2 * d[1][1], q[5]);
        }
    }
}

/*
 * Decode one JPEG byte string (all scans present in it).
 *   coef  optional: receives the coefficient planes
 *   pix   optional: receives H*W*nc bytes, row-major, channel-interleaved
 *   upsample  0 replicate (the contract), 1 triangle + per-plane rounding (comparison only)
 *   idct_direct  1 = evaluate the O(N^4) definition, 0 = separable
 */
static int decode_impl(const uint8_t* jpg, size_t n, int upsample, int idct_direct, int smooth, int16_t* coef, uint8_t* pix) {
    orc_info_t info;
    dec_t* D = (dec_t*)malloc(sizeof(dec_t));
    int rc = walk(jpg, n, D, &info, NULL);
    if (rc) { free(D); return rc; }
    size_t total = 0;
    for (int c = 0; c < info.nc; c++) total += (size_t)info.bw[c] * info.bh[c] * 64;
    int16_t* cbuf = coef ? coef : (int16_t*)malloc(total * sizeof(int16_t));
    rc = walk(jpg, n, D, &info, cbuf);
    if (!rc && (pix || smooth)) {
        for (int c = 0; c < D->nc; c++) if (!D->qdef[D->tq[c]]) rc = ORC_E_FORMAT;
    }
    if (!rc && smooth) smooth_dc_only_components(D);
    if (!rc && pix) {
        double* plane[3] = {0, 0, 0};
        for (int c = 0; c < D->nc; c++) plane[c] = (double*)malloc(sizeof(double) * (size_t)D->bw[c] * D->bh[c] * 64);
        planes_from_coefs(D, idct_direct, plane);
        if (upsample == 1)
            for (int c = 0; c < D->nc; c++) { size_t np = (size_t)D->bw[c] * D->bh[c] * 64; for (size_t i = 0; i < np; i++) plane[c][i] = floor(plane[c][i] + 0.5); }
        for (int y = 0; y < D->H; y++) for (int x = 0; x < D->W; x++) {
            double s[3];
            for (int c = 0; c < D->nc; c++) {
                int pw = D->bw[c] * 8;
                int fx = D->hmax / D->hs[c], fy = D->vmax / D->vs[c];
                if (upsample == 0 || (fx == 1 && fy == 1)) s[c] = plane[c][(size_t)((y * D->vs[c]) / D->vmax) * pw + (x * D->hs[c]) / D->hmax];
                else {
                    int xc = (D->W * D->hs[c] + D->hmax - 1) / D->hmax, yc = (D->H * D->vs[c] + D->vmax - 1) / D->vmax;
                    /* vertical then horizontal triangle on the cropped plane */
                    double col[2]; int xi = fx == 2 ? x >> 1 : x;
                    int xj = fx == 2 ? ((x & 1) ? xi + 1 : xi - 1) : xi;
                    if (xj < 0) xj = 0;
                    if (xj >= xc) xj = xc - 1;
                    int xs[2] = { xi, xj };
                    for (int q = 0; q < 2; q++)
                        col[q] = fy == 2 ? tri(plane[c] + xs[q], yc, pw, y) : plane[c][(size_t)y * pw + xs[q]];
                    s[c] = fx == 2 ? 0.75 * col[0] + 0.25 * col[1] : col[0];
                }
            }
            uint8_t* o = pix + ((size_t)y * D->W + x) * D->nc;
            if (D->nc == 1) o[0] = round_u8(s[0]);
            else {
                double Y = s[0], Cb = s[1] - 128.0, Cr = s[2] - 128.0;
                o[0] = round_u8(Y + 1.402 * Cr);
                o[1] = round_u8(Y - 0.344136 * Cb - 0.714136 * Cr);
                o[2] = round_u8(Y + 1.772 * Cb);
            }
        }
        for (int c = 0; c < D->nc; c++) free(plane[c]);
    }
    if (!coef) free(cbuf);
    free(D);
    return rc;
}
int orc_decode(const uint8_t* jpg, size_t n, int upsample, int idct_direct, int16_t* coef, uint8_t* pix) {
    return decode_impl(jpg, n, upsample, idct_direct, 0, coef, pix);
}
/* The same with the smoothing above (replicated chroma, separable transform); coef, if given, receives the
 * coefficients with the predictions in place. */
int orc_decode_smooth(const uint8_t* jpg, size_t n, int16_t* coef, uint8_t* pix) {
    return decode_impl(jpg, n, 0, 0, 1, coef, pix);
}

/* Convenience for whole records: decode image i at fidelity k straight from the record. */
int orc_decode_record_image(const uint8_t* rec, size_t nbytes, uint32_t i, int k, int upsample, int idct_direct,
                            int16_t* coef, uint8_t* pix) {
    size_t L = 0;
    int rc = orc_reassemble(rec, nbytes, i, k, NULL, 0, &L);
    if (rc) return rc;
    uint8_t* buf = (uint8_t*)malloc(L ? L : 1);
    rc = orc_reassemble(rec, nbytes, i, k, buf, L, &L);
    if (!rc) rc = orc_decode(buf, L, upsample, idct_direct, coef, pix);
    free(buf);
    return rc;
}

int orc_record_image_info(const uint8_t* rec, size_t nbytes, uint32_t i, orc_info_t* info) {
    size_t L = 0;
    int rc = orc_reassemble(rec, nbytes, i, 1, NULL, 0, &L);
    if (rc) return rc;
    uint8_t* buf = (uint8_t*)malloc(L ? L : 1);
    rc = orc_reassemble(rec, nbytes, i, 1, buf, L, &L);
    if (!rc) rc = orc_image_info(buf, L, info);
    free(buf);
    return rc;
}
