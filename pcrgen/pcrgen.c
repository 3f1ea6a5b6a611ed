/*
 * pcrgen -- seeded synthetic input generator for Progressive Compressed Record tests and
 * benchmarks: image synthesis, a JPEG *encoder* (sequential SOF0 and progressive SOF2 with
 * an arbitrary scan script, optimised Huffman tables, optional restart intervals) and the
 * scan splitter used to build records.
 *
 * This module only PRODUCES inputs.  It contains no decoder and is used by neither the CPU
 * oracle nor the GPU library; both merely consume the bytes it writes.  The paper builds its
 * records from progressive files written by a stock transcoder (Section 5, "Encoding"); this
 * file stands in for that tool so that inputs can be made without any dataset.
 *
 * Plain C99, no dependencies beyond libm.  All entry points are re-entrant.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define PI 3.14159265358979323846

/* ------------------------------------------------------------------------------------------
 * Counter-based random numbers: splitmix64 finaliser over (seed, counter).
 * ---------------------------------------------------------------------------------------- */
typedef struct { uint64_t s, c; } rng_t;

static uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static uint64_t rng_u64(rng_t* r) { return mix64(r->s ^ mix64(r->c++)); }
static double rng_unit(rng_t* r) { return (double)(rng_u64(r) >> 11) * (1.0 / 9007199254740992.0); }
static double rng_range(rng_t* r, double a, double b) { return a + (b - a) * rng_unit(r); }
static double rng_normal(rng_t* r) {
    double u1 = rng_unit(r), u2 = rng_unit(r);
    if (u1 < 1e-300) u1 = 1e-300;
    return sqrt(-2.0 * log(u1)) * cos(2.0 * PI * u2);
}

/* ------------------------------------------------------------------------------------------
 * Image synthesis.  kind:
 *   0  sum of 4 random 2-D sinusoids per channel + Gaussian noise(sigma)
 *   1  kind 0 + random filled rectangles
 *   2  "textured": kind 1 + multi-octave value noise (bilinear-interpolated random lattices
 *      with cell sizes 2..64 and amplitude growing with cell size, partly shared by the
 *      channels), which gives the 1/f-like spectrum of photographs
 *   3  heavy-tailed: with probability 0.7 a smooth two-axis gradient, else flat grey +
 *      Gaussian noise(sigma); the draw is part of the seeded stream
 * Output: H x W x C uint8, channel-interleaved.
 * ---------------------------------------------------------------------------------------- */
/* texture constants of kind 2, tuned so that 300..500 px images at quality 90 average about
 * 105 kB with per-scan cumulative sizes near the ratios of the paper's Table 1 (ImageNet row) */
static const double tex_amp = 6.0, tex_slope = 0.6, patch_density = 0.2;

void pcrgen_synth(uint64_t seed, int kind, int W, int H, int C, double sigma, uint8_t* out) {
    rng_t r = { mix64(seed), 0 };
    size_t npx = (size_t)W * H;
    float* plane = (float*)malloc(npx * sizeof(float));
    double* sx = (double*)malloc(sizeof(double) * 2 * (size_t)(W > H ? W : H) * 2);
    double *cxv = sx, *sxv = sx + W, *cyv = sx + 2 * (size_t)(W > H ? W : H), *syv = cyv + H;
    int smooth = 0;
    if (kind == 3) smooth = rng_unit(&r) < 0.7;
    /* rectangles are shared by the channels (position/size) but coloured per channel */
    int nrect = (kind == 1 || kind == 2) ? 3 + (int)(rng_unit(&r) * 6) : 0;
    int rx0[16], ry0[16], rx1[16], ry1[16];
    for (int q = 0; q < nrect; q++) {
        int w = 1 + (int)(rng_unit(&r) * W / 2), h = 1 + (int)(rng_unit(&r) * H / 2);
        rx0[q] = (int)(rng_unit(&r) * (W - w + 1)); ry0[q] = (int)(rng_unit(&r) * (H - h + 1));
        rx1[q] = rx0[q] + w; ry1[q] = ry0[q] + h;
    }
    for (int c = 0; c < C; c++) {
        for (size_t p = 0; p < npx; p++) plane[p] = 128.0f;
        if (kind == 3) {
            if (smooth) {
                double gx = rng_range(&r, -100, 100) / W, gy = rng_range(&r, -100, 100) / H;
                double base = rng_range(&r, 90, 166);
                for (int y = 0; y < H; y++)
                    for (int x = 0; x < W; x++)
                        plane[(size_t)y * W + x] = (float)(base + gx * (x - W / 2) + gy * (y - H / 2));
            }
        } else {
            for (int j = 0; j < 4; j++) {
                double fx = rng_range(&r, 0.5, 6.0) / W * (rng_unit(&r) < 0.5 ? -1 : 1);
                double fy = rng_range(&r, 0.5, 6.0) / H;
                double ph = rng_range(&r, 0, 2 * PI);
                double A = rng_range(&r, 8, 30);
                for (int x = 0; x < W; x++) { cxv[x] = cos(2 * PI * fx * x + ph); sxv[x] = sin(2 * PI * fx * x + ph); }
                for (int y = 0; y < H; y++) { cyv[y] = cos(2 * PI * fy * y); syv[y] = sin(2 * PI * fy * y); }
                for (int y = 0; y < H; y++) {
                    float* row = plane + (size_t)y * W;
                    double cy = cyv[y] * A, sy = syv[y] * A;
                    for (int x = 0; x < W; x++) row[x] += (float)(sxv[x] * cy + cxv[x] * sy);
                }
            }
            if (kind == 2) {
                /* octave o: lattice cell 2^o pixels; the lattice of channel c mixes a field shared
                 * by all channels (seeded per octave) with one of its own */
                for (int o = 1; o <= 6; o++) {
                    int cell = 1 << o, gw = W / cell + 2, gh = H / cell + 2;
                    float* g = (float*)malloc(sizeof(float) * (size_t)gw * gh);
                    rng_t shared = { mix64(seed ^ (0xA5A5ull + (uint64_t)o)), 0 };
                    double A = tex_amp * pow((double)cell, tex_slope);
                    for (int q = 0; q < gw * gh; q++)
                        g[q] = (float)(A * (0.8 * rng_range(&shared, -1, 1) + 0.45 * rng_range(&r, -1, 1)));
                    for (int y = 0; y < H; y++) {
                        int gy = y / cell; float fy = (float)(y % cell) / cell;
                        float* row = plane + (size_t)y * W;
                        for (int x = 0; x < W; x++) {
                            int gx = x / cell; float fx = (float)(x % cell) / cell;
                            const float* q0 = g + (size_t)gy * gw + gx; const float* q1 = q0 + gw;
                            row[x] += (q0[0] * (1 - fx) + q0[1] * fx) * (1 - fy) + (q1[0] * (1 - fx) + q1[1] * fx) * fy;
                        }
                    }
                    free(g);
                }
            }
            if (kind == 2) {
                /* many small high-contrast patches: sparse, large high-frequency coefficients
                 * (edges), the same patch geometry in every channel with a per-channel gain */
                rng_t geo = { mix64(seed ^ 0xEDCEull), 0 };
                long npatch = (long)((double)W * H * patch_density);
                for (long q = 0; q < npatch; q++) {
                    int pw = 2 + (int)(rng_unit(&geo) * 18), ph = 2 + (int)(rng_unit(&geo) * 18);
                    int px = (int)(rng_unit(&geo) * W), py = (int)(rng_unit(&geo) * H);
                    double amp = rng_range(&geo, 15, 70) * (rng_unit(&geo) < 0.5 ? -1 : 1);
                    float a = (float)(amp * rng_range(&r, 0.1, 1.9));
                    for (int y = py; y < py + ph && y < H; y++)
                        for (int x = px; x < px + pw && x < W; x++) plane[(size_t)y * W + x] += a;
                }
            }
            for (int q = 0; q < nrect; q++) {
                float v = (float)rng_range(&r, 20, 235);
                for (int y = ry0[q]; y < ry1[q]; y++)
                    for (int x = rx0[q]; x < rx1[q]; x++) plane[(size_t)y * W + x] = v;
            }
        }
        double sg = (kind == 3 && smooth) ? 0.0 : sigma;
        for (size_t p = 0; p < npx; p++) {
            double v = plane[p];
            if (sg > 0) v += sg * rng_normal(&r);
            v = floor(v + 0.5);
            if (v < 0) v = 0;
            if (v > 255) v = 255;
            out[p * C + c] = (uint8_t)v;
        }
    }
    free(plane); free(sx);
}

/* ------------------------------------------------------------------------------------------
 * Tables.  The two example quantisation tables of the JPEG standard's Annex K, listed in
 * zig-zag order (the order a DQT segment stores them).
 * ---------------------------------------------------------------------------------------- */
static const uint8_t base_q_zz[2][64] = {
  {16, 11, 12, 14, 12, 10, 16, 14, 13, 14, 18, 17, 16, 19, 24, 40, 26, 24, 22, 22, 24, 49, 35, 37,
   29, 40, 58, 51, 61, 60, 57, 51, 56, 55, 64, 72, 92, 78, 64, 68, 87, 69, 55, 56, 80, 109, 81, 87,
   95, 98, 103, 104, 103, 62, 77, 113, 121, 112, 100, 120, 92, 101, 103, 99},
  {17, 18, 18, 24, 21, 24, 47, 26, 26, 47, 99, 66, 56, 66, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99,
   99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99,
   99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99, 99}
};

/* zig-zag position -> natural (row-major) index, generated by walking the anti-diagonals */
static void make_zigzag(int zz[64]) {
    int n = 0;
    for (int d = 0; d < 15; d++) {
        if (d & 1) { for (int y = (d < 8 ? 0 : d - 7); y <= (d < 8 ? d : 7); y++) zz[n++] = y * 8 + (d - y); }
        else       { for (int x = (d < 8 ? 0 : d - 7); x <= (d < 8 ? d : 7); x++) zz[n++] = (d - x) * 8 + x; }
    }
}

/* quality -> quantisation table in zig-zag order (linear scaling of the base table) */
void pcrgen_quant_table(int which, int quality, uint16_t out_zz[64]) {
    if (quality < 1) quality = 1;
    if (quality > 100) quality = 100;
    int scale = quality < 50 ? 5000 / quality : 200 - 2 * quality;
    for (int i = 0; i < 64; i++) {
        int v = (base_q_zz[which][i] * scale + 50) / 100;
        if (v < 1) v = 1;
        if (v > 255) v = 255;
        out_zz[i] = (uint16_t)v;
    }
}

/* ------------------------------------------------------------------------------------------
 * Byte sink with JPEG stuffing.
 * ---------------------------------------------------------------------------------------- */
typedef struct { uint8_t* p; size_t n, cap; int overflow; uint32_t acc; int nacc; } sink_t;
static void put_raw(sink_t* s, int b) { if (s->n < s->cap) s->p[s->n++] = (uint8_t)b; else s->overflow = 1; }
static void put16(sink_t* s, int v) { put_raw(s, v >> 8); put_raw(s, v & 255); }
static void put_bits(sink_t* s, uint32_t bits, int n) {     /* n <= 16 */
    if (!n) return;
    s->acc = (s->acc << n) | (bits & ((1u << n) - 1)); s->nacc += n;
    while (s->nacc >= 8) {
        int b = (s->acc >> (s->nacc - 8)) & 255;
        put_raw(s, b); if (b == 255) put_raw(s, 0);
        s->nacc -= 8;
    }
}
static void flush_bits(sink_t* s) {                          /* pad with 1-bits */
    if (s->nacc) put_bits(s, (1u << (8 - s->nacc)) - 1, 8 - s->nacc);
    s->acc = 0; s->nacc = 0;
}

/* ------------------------------------------------------------------------------------------
 * Token stream of one scan: Huffman symbols (with appended raw bits), bare raw bits, restarts.
 * ---------------------------------------------------------------------------------------- */
typedef struct { int16_t sym; uint8_t tbl; uint8_t nbits; uint32_t bits; } tok_t;  /* sym<0: raw only; tbl 255: RST */
typedef struct { tok_t* t; size_t n, cap; } toks_t;
static void tok_push(toks_t* T, int sym, int tbl, uint32_t bits, int nbits) {
    if (T->n == T->cap) { T->cap = T->cap ? T->cap * 2 : 4096; T->t = (tok_t*)realloc(T->t, T->cap * sizeof(tok_t)); }
    tok_t k; k.sym = (int16_t)sym; k.tbl = (uint8_t)tbl; k.nbits = (uint8_t)nbits; k.bits = bits;
    T->t[T->n++] = k;
}

/* Optimal prefix code lengths limited to 16 bits, with one reserved leaf so that no real
 * symbol receives the all-ones code word.  freq[256] -> BITS[1..16], HUFFVAL (returns count). */
static int build_huffman(const long freq_in[256], uint8_t bits[17], uint8_t vals[256]) {
    int len[257]; int parent[2 * 257]; long w[2 * 257]; int alive[2 * 257];
    int ids[257], m = 0;
    for (int i = 0; i < 256; i++) if (freq_in[i] > 0) ids[m++] = i;
    memset(bits, 0, 17);
    if (m == 0) return 0;
    int nleaf = m + 1;                       /* + reserved leaf, weight below every real one */
    int nn = nleaf;
    for (int i = 0; i < m; i++) { w[i] = freq_in[ids[i]] * 2; alive[i] = 1; parent[i] = -1; }
    w[m] = 1; alive[m] = 1; parent[m] = -1;
    while (1) {
        int a = -1, b = -1;
        for (int i = 0; i < nn; i++) if (alive[i]) {
            if (a < 0 || w[i] < w[a]) { b = a; a = i; }
            else if (b < 0 || w[i] < w[b]) b = i;
        }
        if (b < 0) break;
        w[nn] = w[a] + w[b]; alive[nn] = 1; parent[nn] = -1; alive[a] = alive[b] = 0; parent[a] = parent[b] = nn; nn++;
    }
    int maxlen = 0;
    for (int i = 0; i < nleaf; i++) { int l = 0, p = i; while (parent[p] >= 0) { p = parent[p]; l++; } if (l == 0) l = 1; len[i] = l; if (l > maxlen) maxlen = l; }
    /* length limiting: count per length, then repeatedly move a pair up (standard rebalancing
     * of the length histogram; keeps the Kraft sum at 1) */
    int cnt[320]; memset(cnt, 0, sizeof cnt);
    for (int i = 0; i < nleaf; i++) cnt[len[i]]++;
    for (int l = maxlen; l > 16; l--) {
        while (cnt[l] > 0) {
            int j = l - 2; while (cnt[j] == 0) j--;
            cnt[l] -= 2; cnt[l - 1] += 1; cnt[j + 1] += 2; cnt[j] -= 1;
        }
    }
    /* assign lengths back: more frequent symbols get shorter codes; reserved leaf is last */
    int order[257];
    for (int i = 0; i < nleaf; i++) order[i] = i;
    for (int i = 1; i < nleaf; i++) {        /* insertion sort by weight desc, stable */
        int o = order[i], j = i - 1;
        while (j >= 0 && w[order[j]] < w[o]) { order[j + 1] = order[j]; j--; }
        order[j + 1] = o;
    }
    int k = 0, nv = 0;
    for (int l = 1; l <= 16; l++)
        for (int q = 0; q < cnt[l]; q++) {
            int leaf = order[k++];
            if (leaf == m) continue;         /* reserved leaf takes the last (all-ones) code */
            bits[l]++; vals[nv++] = (uint8_t)ids[leaf];
        }
    return nv;
}

typedef struct { uint16_t code[256]; uint8_t len[256]; } hcode_t;
static void make_codes(const uint8_t bits[17], const uint8_t* vals, hcode_t* h) {
    memset(h, 0, sizeof *h);
    int code = 0, k = 0;
    for (int l = 1; l <= 16; l++) {
        for (int i = 0; i < bits[l]; i++) { h->code[vals[k]] = (uint16_t)code; h->len[vals[k]] = (uint8_t)l; code++; k++; }
        code <<= 1;
    }
}

/* ------------------------------------------------------------------------------------------
 * Frame description shared by the scan encoders.
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    int W, H, nc;
    int hs[3], vs[3];            /* sampling factors */
    int hmax, vmax, mcux, mcuy;
    int bw[3], bh[3];            /* allocated (MCU padded) block grid */
    int cw[3], ch[3];            /* blocks covering the component's own samples */
    const int16_t* coef[3];      /* [bh][bw][64] natural order */
    int zz[64];
} frame_t;

static void frame_init(frame_t* F, int W, int H, int nc, int hsub, int vsub) {
    memset(F, 0, sizeof *F);
    F->W = W; F->H = H; F->nc = nc;
    for (int c = 0; c < nc; c++) { F->hs[c] = (c == 0 && nc == 3) ? hsub : 1; F->vs[c] = (c == 0 && nc == 3) ? vsub : 1; }
    F->hmax = nc == 3 ? hsub : 1; F->vmax = nc == 3 ? vsub : 1;
    F->mcux = (W + 8 * F->hmax - 1) / (8 * F->hmax); F->mcuy = (H + 8 * F->vmax - 1) / (8 * F->vmax);
    for (int c = 0; c < nc; c++) {
        F->bw[c] = F->mcux * F->hs[c]; F->bh[c] = F->mcuy * F->vs[c];
        int xc = (W * F->hs[c] + F->hmax - 1) / F->hmax, yc = (H * F->vs[c] + F->vmax - 1) / F->vmax;
        F->cw[c] = (xc + 7) / 8; F->ch[c] = (yc + 7) / 8;
    }
    make_zigzag(F->zz);
}

size_t pcrgen_plane_blocks(int W, int H, int nc, int hsub, int vsub, int c) {
    frame_t F; frame_init(&F, W, H, nc, hsub, vsub);
    return (size_t)F.bw[c] * F.bh[c];
}

static int bitlen(int v) { int n = 0; while (v) { n++; v >>= 1; } return n; }

/* ---- end-of-band run bookkeeping shared by the AC scans ---- */
typedef struct {
    toks_t* T; int actbl; int eobrun;
    uint8_t* pend; size_t npend, cappend;     /* correction bits waiting behind the EOB run */
} acstate_t;
static void pend_push(acstate_t* S, int bit) {
    if (S->npend == S->cappend) { S->cappend = S->cappend ? S->cappend * 2 : 1024; S->pend = (uint8_t*)realloc(S->pend, S->cappend); }
    S->pend[S->npend++] = (uint8_t)bit;
}
static void emit_bitlist(toks_t* T, const uint8_t* b, size_t n) {
    size_t i = 0;
    while (i < n) {
        uint32_t v = 0; int k = 0;
        while (k < 16 && i < n) { v = (v << 1) | b[i++]; k++; }
        tok_push(T, -1, 0, v, k);
    }
}
static void flush_eobrun(acstate_t* S) {
    if (S->eobrun > 0) {
        int nb = bitlen(S->eobrun) - 1;
        tok_push(S->T, nb << 4, S->actbl, (uint32_t)(S->eobrun - (1 << nb)), nb);
        S->eobrun = 0;
    }
    emit_bitlist(S->T, S->pend, S->npend); S->npend = 0;
}

static void enc_ac_first_block(acstate_t* S, const int16_t* blk, const int* zz, int Ss, int Se, int Al) {
    int r = 0;
    for (int k = Ss; k <= Se; k++) {
        int c = blk[zz[k]];
        int a = (c < 0 ? -c : c) >> Al;
        if (a == 0) { r++; continue; }
        flush_eobrun(S);
        while (r > 15) { tok_push(S->T, 0xF0, S->actbl, 0, 0); r -= 16; }
        int nb = bitlen(a);
        int v = c < 0 ? -a : a;
        uint32_t extra = (uint32_t)(v < 0 ? v - 1 : v) & ((1u << nb) - 1);
        tok_push(S->T, (r << 4) | nb, S->actbl, extra, nb);
        r = 0;
    }
    if (r > 0) { S->eobrun++; if (S->eobrun == 0x7FFF) flush_eobrun(S); }
}

static void enc_ac_refine_block(acstate_t* S, const int16_t* blk, const int* zz, int Ss, int Se, int Al) {
    int a[64], eobpos = -1;
    for (int k = Ss; k <= Se; k++) {
        int c = blk[zz[k]];
        a[k] = (c < 0 ? -c : c) >> Al;
        if (a[k] == 1) eobpos = k;             /* last coefficient that becomes non-zero now */
    }
    uint8_t br[64]; int nbr = 0, r = 0;
    for (int k = Ss; k <= Se; k++) {
        if (a[k] == 0) { r++; continue; }
        while (r > 15 && k <= eobpos) {
            flush_eobrun(S);
            tok_push(S->T, 0xF0, S->actbl, 0, 0); r -= 16;
            emit_bitlist(S->T, br, nbr); nbr = 0;
        }
        if (a[k] > 1) { br[nbr++] = (uint8_t)(a[k] & 1); continue; }   /* already non-zero: correction bit */
        flush_eobrun(S);
        tok_push(S->T, (r << 4) | 1, S->actbl, blk[zz[k]] < 0 ? 0u : 1u, 1);
        emit_bitlist(S->T, br, nbr); nbr = 0; r = 0;
    }
    if (r > 0 || nbr > 0) {
        S->eobrun++;
        for (int i = 0; i < nbr; i++) pend_push(S, br[i]);
        if (S->eobrun == 0x7FFF) flush_eobrun(S);
    }
}

/* One scan -> tokens.  comps[]: component indices; interleaved if ns > 1. */
static void scan_tokens(const frame_t* F, int ns, const int* comps, int Ss, int Se, int Ah, int Al,
                        int Ri, int sequential, toks_t* T) {
    int pred[3] = {0, 0, 0};
    acstate_t S; memset(&S, 0, sizeof S); S.T = T;
    long mcu_total, mcu_w;
    if (ns > 1) { mcu_w = F->mcux; mcu_total = (long)F->mcux * F->mcuy; }
    else { mcu_w = F->cw[comps[0]]; mcu_total = (long)F->cw[comps[0]] * F->ch[comps[0]]; }
    int rstn = 0;
    for (long m = 0; m < mcu_total; m++) {
        if (Ri > 0 && m > 0 && m % Ri == 0) {
            flush_eobrun(&S);
            tok_push(T, rstn, 255, 0, 0); rstn = (rstn + 1) & 7;
            pred[0] = pred[1] = pred[2] = 0;
        }
        long my = m / mcu_w, mx = m % mcu_w;
        for (int ci = 0; ci < ns; ci++) {
            int c = comps[ci];
            int nbx = ns > 1 ? F->hs[c] : 1, nby = ns > 1 ? F->vs[c] : 1;
            for (int by = 0; by < nby; by++) for (int bx = 0; bx < nbx; bx++) {
                long brow = ns > 1 ? my * F->vs[c] + by : my, bcol = ns > 1 ? mx * F->hs[c] + bx : mx;
                const int16_t* blk = F->coef[c] + ((size_t)brow * F->bw[c] + bcol) * 64;
                int dctbl = c == 0 ? 0 : 1, actbl = c == 0 ? 2 : 3;
                S.actbl = actbl;
                if (sequential) {
                    int d = blk[0] - pred[c]; pred[c] = blk[0];
                    int ad = d < 0 ? -d : d, nb = bitlen(ad);
                    tok_push(T, nb, dctbl, (uint32_t)(d < 0 ? d - 1 : d) & ((1u << nb) - 1), nb);
                    int r = 0;
                    for (int k = 1; k < 64; k++) {
                        int v = blk[F->zz[k]];
                        if (v == 0) { r++; continue; }
                        while (r > 15) { tok_push(T, 0xF0, actbl, 0, 0); r -= 16; }
                        int av = v < 0 ? -v : v, nbv = bitlen(av);
                        tok_push(T, (r << 4) | nbv, actbl, (uint32_t)(v < 0 ? v - 1 : v) & ((1u << nbv) - 1), nbv);
                        r = 0;
                    }
                    if (r > 0) tok_push(T, 0x00, actbl, 0, 0);
                } else if (Ss == 0) {
                    if (Ah == 0) {
                        int v = blk[0] >> Al;                 /* arithmetic shift: DC point transform */
                        int d = v - pred[c]; pred[c] = v;
                        int ad = d < 0 ? -d : d, nb = bitlen(ad);
                        tok_push(T, nb, dctbl, (uint32_t)(d < 0 ? d - 1 : d) & ((1u << nb) - 1), nb);
                    } else {
                        tok_push(T, -1, 0, (uint32_t)((blk[0] >> Al) & 1), 1);
                    }
                } else if (Ah == 0) enc_ac_first_block(&S, blk, F->zz, Ss, Se, Al);
                else enc_ac_refine_block(&S, blk, F->zz, Ss, Se, Al);
            }
        }
    }
    flush_eobrun(&S);
    free(S.pend);
}

static void write_dht(sink_t* s, int tc, int th, const uint8_t bits[17], const uint8_t* vals, int nv) {
    put16(s, 0xFFC4); put16(s, 2 + 1 + 16 + nv); put_raw(s, (tc << 4) | th);
    for (int l = 1; l <= 16; l++) put_raw(s, bits[l]);
    for (int i = 0; i < nv; i++) put_raw(s, vals[i]);
}

/* script entry: {ns, c0, c1, c2, Ss, Se, Ah, Al} */
#define SCRIPT_STRIDE 8

static const int script_color10[10 * SCRIPT_STRIDE] = {
    3, 0, 1, 2, 0, 0, 0, 1,
    1, 0, 0, 0, 1, 5, 0, 2,
    1, 2, 0, 0, 1, 63, 0, 1,
    1, 1, 0, 0, 1, 63, 0, 1,
    1, 0, 0, 0, 6, 63, 0, 2,
    1, 0, 0, 0, 1, 63, 2, 1,
    3, 0, 1, 2, 0, 0, 1, 0,
    1, 2, 0, 0, 1, 63, 1, 0,
    1, 1, 0, 0, 1, 63, 1, 0,
    1, 0, 0, 0, 1, 63, 1, 0 };
static const int script_gray6[6 * SCRIPT_STRIDE] = {
    1, 0, 0, 0, 0, 0, 0, 1,
    1, 0, 0, 0, 1, 5, 0, 2,
    1, 0, 0, 0, 6, 63, 0, 2,
    1, 0, 0, 0, 1, 63, 2, 1,
    1, 0, 0, 0, 0, 0, 1, 0,
    1, 0, 0, 0, 1, 63, 1, 0 };

/*
 * Entropy-code coefficient planes into a JPEG file.
 *   coef        concatenated planes c = 0..nc-1, each [bh_c][bw_c][64] int16, natural order
 *   qzz         nc>1 ? 2 : 1 tables x 64, zig-zag order (table 0 for component 0, 1 for the rest)
 *   script      n_scans x 8 ints, or NULL with n_scans = 0 for the default progressive script
 *               (10 scans for 3 components, 6 for one); n_scans = -1 -> sequential SOF0 file
 *   restart     0 none; 1 = one restart interval per MCU row of each scan; >1 = Ri in MCUs
 * Returns bytes written, 0 on overflow.
 */
size_t pcrgen_encode_coefs(const int16_t* coef, int W, int H, int nc, int hsub, int vsub,
                           const uint16_t* qzz, const int* script, int n_scans, int restart,
                           uint8_t* out, size_t cap) {
    frame_t F; frame_init(&F, W, H, nc, hsub, vsub);
    size_t o = 0;
    for (int c = 0; c < nc; c++) { F.coef[c] = coef + o; o += (size_t)F.bw[c] * F.bh[c] * 64; }
    sink_t s; memset(&s, 0, sizeof s); s.p = out; s.cap = cap;
    int sequential = n_scans < 0;
    static const int seq_gray[SCRIPT_STRIDE] = {1, 0, 0, 0, 0, 63, 0, 0};
    static const int seq_col[SCRIPT_STRIDE] = {3, 0, 1, 2, 0, 63, 0, 0};
    if (sequential) { script = nc == 3 ? seq_col : seq_gray; n_scans = 1; }
    else if (!script || n_scans == 0) { script = nc == 3 ? script_color10 : script_gray6; n_scans = nc == 3 ? 10 : 6; }

    put16(&s, 0xFFD8);
    put16(&s, 0xFFE0); put16(&s, 16); { const char* j = "JFIF"; for (int i = 0; i < 5; i++) put_raw(&s, j[i]); }
    put16(&s, 0x0101); put_raw(&s, 0); put16(&s, 1); put16(&s, 1); put_raw(&s, 0); put_raw(&s, 0);
    int nq = nc == 3 ? 2 : 1;
    for (int t = 0; t < nq; t++) {
        put16(&s, 0xFFDB); put16(&s, 67); put_raw(&s, t);
        for (int i = 0; i < 64; i++) put_raw(&s, qzz[t * 64 + i] > 255 ? 255 : qzz[t * 64 + i]);
    }
    put16(&s, sequential ? 0xFFC0 : 0xFFC2); put16(&s, 8 + 3 * nc); put_raw(&s, 8); put16(&s, H); put16(&s, W); put_raw(&s, nc);
    for (int c = 0; c < nc; c++) { put_raw(&s, c + 1); put_raw(&s, (F.hs[c] << 4) | F.vs[c]); put_raw(&s, c == 0 ? 0 : 1); }

    int cur_ri = 0;
    toks_t T; memset(&T, 0, sizeof T);
    for (int sc = 0; sc < n_scans; sc++) {
        const int* e = script + sc * SCRIPT_STRIDE;
        int ns = e[0]; const int* comps = e + 1; int Ss = e[4], Se = e[5], Ah = e[6], Al = e[7];
        int Ri = 0;
        if (restart == 1) Ri = ns > 1 ? F.mcux : F.cw[comps[0]];
        else if (restart > 1) Ri = restart;
        T.n = 0;
        scan_tokens(&F, ns, comps, Ss, Se, Ah, Al, Ri, sequential, &T);
        long freq[4][256]; memset(freq, 0, sizeof freq);
        for (size_t i = 0; i < T.n; i++) if (T.t[i].sym >= 0 && T.t[i].tbl < 4) freq[T.t[i].tbl][T.t[i].sym]++;
        hcode_t hc[4];
        for (int t = 0; t < 4; t++) {
            uint8_t bits[17], vals[256];
            int nv = build_huffman(freq[t], bits, vals);
            if (nv == 0) continue;
            write_dht(&s, t >> 1, t & 1, bits, vals, nv);
            make_codes(bits, vals, &hc[t]);
        }
        if (Ri != cur_ri) { put16(&s, 0xFFDD); put16(&s, 4); put16(&s, Ri); cur_ri = Ri; }
        put16(&s, 0xFFDA); put16(&s, 6 + 2 * ns); put_raw(&s, ns);
        for (int ci = 0; ci < ns; ci++) { int c = comps[ci]; put_raw(&s, c + 1); put_raw(&s, c == 0 ? 0x00 : 0x11); }
        put_raw(&s, Ss); put_raw(&s, Se); put_raw(&s, (Ah << 4) | Al);
        for (size_t i = 0; i < T.n; i++) {
            tok_t k = T.t[i];
            if (k.tbl == 255) { flush_bits(&s); put_raw(&s, 0xFF); put_raw(&s, 0xD0 + k.sym); continue; }
            if (k.sym >= 0) put_bits(&s, hc[k.tbl].code[k.sym], hc[k.tbl].len[k.sym]);
            put_bits(&s, k.bits, k.nbits);
        }
        flush_bits(&s);
    }
    free(T.t);
    put16(&s, 0xFFD9);
    return s.overflow ? 0 : s.n;
}

/* ------------------------------------------------------------------------------------------
 * Pixels -> quantised coefficient planes (colour transform, box down-sampling, edge
 * replication to the MCU grid, forward DCT, rounding division).
 * ---------------------------------------------------------------------------------------- */
void pcrgen_pixels_to_coefs(const uint8_t* pix, int W, int H, int nc, int hsub, int vsub,
                            const uint16_t* qzz, int16_t* coef) {
    frame_t F; frame_init(&F, W, H, nc, hsub, vsub);
    double cs[8][8];
    for (int u = 0; u < 8; u++) for (int x = 0; x < 8; x++) cs[u][x] = (u == 0 ? sqrt(0.5) : 1.0) * 0.5 * cos((2 * x + 1) * u * PI / 16);
    size_t o = 0;
    for (int c = 0; c < nc; c++) {
        int pw = F.bw[c] * 8, ph = F.bh[c] * 8;
        int sx = F.hmax / F.hs[c], sy = F.vmax / F.vs[c];
        int xc = (W * F.hs[c] + F.hmax - 1) / F.hmax, yc = (H * F.vs[c] + F.vmax - 1) / F.vmax;
        float* pl = (float*)malloc(sizeof(float) * (size_t)pw * ph);
        for (int y = 0; y < ph; y++) for (int x = 0; x < pw; x++) {
            int yy = y < yc ? y : yc - 1, xx = x < xc ? x : xc - 1;
            double acc = 0;
            for (int dy = 0; dy < sy; dy++) for (int dx = 0; dx < sx; dx++) {
                int py = yy * sy + dy, px = xx * sx + dx;
                if (py >= H) py = H - 1;
                if (px >= W) px = W - 1;
                const uint8_t* p = pix + ((size_t)py * W + px) * nc;
                double v;
                if (nc == 1) v = p[0];
                else if (c == 0) v = 0.299 * p[0] + 0.587 * p[1] + 0.114 * p[2];
                else if (c == 1) v = -0.168736 * p[0] - 0.331264 * p[1] + 0.5 * p[2] + 128;
                else v = 0.5 * p[0] - 0.418688 * p[1] - 0.081312 * p[2] + 128;
                acc += v;
            }
            pl[(size_t)y * pw + x] = (float)(acc / (sx * sy) - 128.0);
        }
        const uint16_t* q = qzz + (c == 0 ? 0 : 64);
        for (int by = 0; by < F.bh[c]; by++) for (int bx = 0; bx < F.bw[c]; bx++) {
            double t[8][8], g[8][8];
            for (int y = 0; y < 8; y++) for (int u = 0; u < 8; u++) {
                double a = 0; for (int x = 0; x < 8; x++) a += cs[u][x] * pl[(size_t)(by * 8 + y) * pw + bx * 8 + x];
                t[y][u] = a;
            }
            for (int v = 0; v < 8; v++) for (int u = 0; u < 8; u++) {
                double a = 0; for (int y = 0; y < 8; y++) a += cs[v][y] * t[y][u];
                g[v][u] = a;
            }
            int16_t* blk = coef + o + ((size_t)by * F.bw[c] + bx) * 64;
            for (int k = 0; k < 64; k++) {
                int nat = F.zz[k]; double val = g[nat >> 3][nat & 7] / q[k];
                blk[nat] = (int16_t)(val < 0 ? -floor(-val + 0.5) : floor(val + 0.5));
            }
        }
        free(pl);
        o += (size_t)F.bw[c] * F.bh[c] * 64;
    }
}

size_t pcrgen_encode_pixels(const uint8_t* pix, int W, int H, int nc, int hsub, int vsub, int quality,
                            const int* script, int n_scans, int restart, uint8_t* out, size_t cap,
                            int16_t* coef_out /* optional, all planes */) {
    frame_t F; frame_init(&F, W, H, nc, hsub, vsub);
    size_t nb = 0; for (int c = 0; c < nc; c++) nb += (size_t)F.bw[c] * F.bh[c];
    uint16_t q[128];
    pcrgen_quant_table(0, quality, q); pcrgen_quant_table(1, quality, q + 64);
    int16_t* coef = coef_out ? coef_out : (int16_t*)malloc(nb * 64 * sizeof(int16_t));
    pcrgen_pixels_to_coefs(pix, W, H, nc, hsub, vsub, q, coef);
    size_t n = pcrgen_encode_coefs(coef, W, H, nc, hsub, vsub, q, script, n_scans, restart, out, cap);
    if (!coef_out) free(coef);
    return n;
}

/* synth + encode in one call (what the benchmark uses; keeps pixels out of Python) */
size_t pcrgen_make_jpeg(uint64_t seed, int kind, int W, int H, int nc, double sigma, int hsub, int vsub,
                        int quality, int restart, uint8_t* out, size_t cap) {
    uint8_t* pix = (uint8_t*)malloc((size_t)W * H * nc);
    pcrgen_synth(seed, kind, W, H, nc, sigma, pix);
    size_t n = pcrgen_encode_pixels(pix, W, H, nc, hsub, vsub, quality, NULL, 0, restart, out, cap, NULL);
    free(pix);
    return n;
}

/* Work accounting for benchmarks: the number of Huffman-coded symbols in every scan of the file pcrgen_make_jpeg
 * (sequential = 0) or pcrgen_make_jpeg_sequential (1) writes for the same arguments -- the symbols a decoder has to
 * decode one after the other.  Bits appended to a symbol and DC refinement bits are not symbols.  Returns the number
 * of scans (counts[0 .. scans-1] filled), or -1 if max_scans is too small. */
int pcrgen_symbol_counts(uint64_t seed, int kind, int W, int H, int nc, double sigma, int hsub, int vsub, int quality,
                         int restart, int sequential, uint64_t* counts, int max_scans) {
    frame_t F; frame_init(&F, W, H, nc, hsub, vsub);
    const int* script = sequential ? NULL : (nc == 3 ? script_color10 : script_gray6);
    static const int seq_gray[SCRIPT_STRIDE] = {1, 0, 0, 0, 0, 63, 0, 0};
    static const int seq_col[SCRIPT_STRIDE] = {3, 0, 1, 2, 0, 63, 0, 0};
    int n_scans = sequential ? 1 : (nc == 3 ? 10 : 6);
    if (sequential) script = nc == 3 ? seq_col : seq_gray;
    if (n_scans > max_scans) return -1;
    size_t nb = 0; for (int c = 0; c < nc; c++) nb += (size_t)F.bw[c] * F.bh[c];
    uint8_t* pix = (uint8_t*)malloc((size_t)W * H * nc);
    int16_t* coef = (int16_t*)malloc(nb * 64 * sizeof(int16_t));
    uint16_t q[128];
    pcrgen_quant_table(0, quality, q); pcrgen_quant_table(1, quality, q + 64);
    pcrgen_synth(seed, kind, W, H, nc, sigma, pix);
    pcrgen_pixels_to_coefs(pix, W, H, nc, hsub, vsub, q, coef);
    size_t o = 0;
    for (int c = 0; c < nc; c++) { F.coef[c] = coef + o; o += (size_t)F.bw[c] * F.bh[c] * 64; }
    toks_t T; memset(&T, 0, sizeof T);
    for (int sc = 0; sc < n_scans; sc++) {
        const int* e = script + sc * SCRIPT_STRIDE;
        int ns = e[0]; const int* comps = e + 1;
        int Ri = 0;
        if (restart == 1) Ri = ns > 1 ? F.mcux : F.cw[comps[0]];
        else if (restart > 1) Ri = restart;
        T.n = 0;
        scan_tokens(&F, ns, comps, e[4], e[5], e[6], e[7], Ri, sequential, &T);
        uint64_t cnt = 0;
        for (size_t i = 0; i < T.n; i++) if (T.t[i].sym >= 0 && T.t[i].tbl < 4) cnt++;
        counts[sc] = cnt;
    }
    free(T.t); free(coef); free(pix);
    return n_scans;
}

/* the same image as a sequential (baseline) file */
size_t pcrgen_make_jpeg_sequential(uint64_t seed, int kind, int W, int H, int nc, double sigma, int hsub, int vsub,
                                   int quality, int restart, uint8_t* out, size_t cap) {
    uint8_t* pix = (uint8_t*)malloc((size_t)W * H * nc);
    pcrgen_synth(seed, kind, W, H, nc, sigma, pix);
    size_t n = pcrgen_encode_pixels(pix, W, H, nc, hsub, vsub, quality, NULL, -1, restart, out, cap, NULL);
    free(pix);
    return n;
}

/* ------------------------------------------------------------------------------------------
 * Scan splitter (paper Section 5, "Encoding": locate the markers that end each scan).
 * After every SOS header the entropy-coded data runs to the first 0xFF that is followed by
 * something other than 0x00, 0xD0..0xD7 or another 0xFF; that position ends the scan's region.
 * The last region runs to the end of the file.  Returns the number of scans, writes the end
 * offset of each region (ends[n-1] == nbytes), or -1 if the file is not well formed.
 * ---------------------------------------------------------------------------------------- */
int pcrgen_split_scans(const uint8_t* d, size_t nbytes, uint64_t* ends, int max_ends) {
    if (nbytes < 4 || d[0] != 0xFF || d[1] != 0xD8) return -1;
    size_t p = 2; int n = 0;
    while (p + 4 <= nbytes) {
        if (d[p] != 0xFF) return -1;
        int m = d[p + 1];
        if (m == 0xFF) { p++; continue; }
        if (m == 0xD9) break;
        size_t L = ((size_t)d[p + 2] << 8) | d[p + 3];
        if (p + 2 + L > nbytes) return -1;
        p += 2 + L;
        if (m != 0xDA) continue;
        while (1) {
            while (p < nbytes && d[p] != 0xFF) p++;
            if (p + 1 >= nbytes) return -1;
            int x = d[p + 1];
            if (x == 0x00 || (x >= 0xD0 && x <= 0xD7)) { p += 2; continue; }
            if (x == 0xFF) {                      /* fill bytes: region ends at the first FF of the run */
                size_t q = p; while (q < nbytes && d[q] == 0xFF) q++;
                if (q >= nbytes) return -1;
                if (d[q] == 0x00 || (d[q] >= 0xD0 && d[q] <= 0xD7)) { p = q + 1; continue; }
            }
            break;
        }
        if (n >= max_ends) return -1;
        ends[n++] = p;
    }
    if (n == 0) return -1;
    ends[n - 1] = nbytes;
    return n;
}
