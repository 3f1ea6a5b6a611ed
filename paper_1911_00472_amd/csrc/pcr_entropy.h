// Progressive-JPEG entropy decoding for one independently decodable unit (a restart interval
// of one scan of one image), written so that the same code runs in a gfx950 lane and on the
// host.  Decoding follows the JPEG progressive mode (spectral selection + successive
// approximation) that the paper's records are made of (Section 2, "Progressive Image
// Compression"; Section 3: scan k of an image is usable once scans 1..k have been read).
//
// Input is the *unstuffed* entropy-coded data of the unit (FF 00 -> FF, restart markers
// removed); a unit never reads a bit past its end: doing so is a data error, not a guess.
//
// AC refinement is decoded against a 64-bit "already non-zero" mask per block (zig-zag bit
// order) instead of against the coefficients themselves: the serial decoder only finds
// where new coefficients go, which signs they get, and the string of correction bits; the
// arithmetic on the coefficients happens later in a data-parallel pass (refine_apply).
#pragma once
#include "pcr_common.h"

namespace pcr {

// ---------------------------------------------------------------------------------------
// Huffman table: 8-bit look-ahead table plus canonical limits for the longer codes.
// ---------------------------------------------------------------------------------------
struct HuffTab {
    uint16_t lut[256];          // (length << 8) | symbol for codes of <= 8 bits, 0 otherwise
    uint32_t limit[17];         // limit[L]: first 16-bit-left-aligned code value NOT of length <= L
    int32_t base[17];           // symbol index = base[L] + (code16 >> (16 - L))
    uint8_t huffval[256];
};

// Build from a DHT payload: 16 counts followed by the symbols in code order.  Codes of each
// length are consecutive integers in symbol order; moving to the next length doubles the code.
PCR_HD void hufftab_build(HuffTab* t, const uint8_t* bits_vals) {
    for (int i = 0; i < 256; i++) t->lut[i] = 0;
    uint32_t code = 0; int k = 0;
    for (int L = 1; L <= 16; L++) {
        int cnt = bits_vals[L - 1];
        t->base[L] = k - (int)code;
        for (int j = 0; j < cnt; j++) {
            if (k < 256) {
                uint8_t sym = bits_vals[16 + k];
                t->huffval[k] = sym;
                if (L <= 8) {
                    uint32_t first = code << (8 - L);
                    uint32_t span = 1u << (8 - L);
                    for (uint32_t e = 0; e < span && first + e < 256; e++) t->lut[first + e] = (uint16_t)((L << 8) | sym);
                }
            }
            code++; k++;
        }
        uint64_t lim = (uint64_t)code << (16 - L);
        t->limit[L] = lim > 65536 ? 65536u : (uint32_t)lim;
        code <<= 1;
    }
}

// ---------------------------------------------------------------------------------------
// Bit reader over unstuffed bytes [p, p + nbytes).  The accumulator holds `cnt` valid bits
// left-aligned in 64 bits.  Bytes past the end read as 0xFF (the padding an encoder
// writes); `overrun()` tells whether more bits were consumed than the unit holds.
// ---------------------------------------------------------------------------------------
struct BitReader {
    const uint8_t* p;
    uint32_t nbytes, pos;       // pos: next byte to load
    uint64_t acc;
    int32_t cnt;
    int64_t consumed;           // bits consumed so far

    PCR_HD void init(const uint8_t* data, uint32_t n) { p = data; nbytes = n; pos = 0; acc = 0; cnt = 0; consumed = 0; refill(); }
    PCR_HD void refill() {
        while (cnt <= 32) {
            uint32_t w = 0;
            for (int j = 0; j < 4; j++) { uint32_t b = (pos + j < nbytes) ? p[pos + j] : 0xFFu; w = (w << 8) | b; }
            pos += 4;
            acc |= (uint64_t)w << (32 - cnt);
            cnt += 32;
        }
    }
    PCR_HD uint32_t peek(int n) const { return (uint32_t)(acc >> (64 - n)); }        // 1 <= n <= 32
    PCR_HD void skip(int n) { acc <<= n; cnt -= n; consumed += n; }
    PCR_HD uint32_t get(int n) {                                                      // 0 <= n <= 32, cnt >= n
        if (n == 0) return 0;
        uint32_t v = peek(n); skip(n); return v;
    }
    PCR_HD bool overrun() const { return consumed > (int64_t)nbytes * 8; }
};

// Decode one Huffman symbol; needs >= 16 valid bits.  Returns -1 for a code that is not in the table.
PCR_HD int huff_decode(BitReader* br, const HuffTab* t) {
    uint32_t e = t->lut[br->peek(8)];
    if (e) { br->skip((int)(e >> 8)); return (int)(e & 255); }
    uint32_t c16 = br->peek(16);
    for (int L = 9; L <= 16; L++) {
        if (c16 < t->limit[L]) {
            int idx = t->base[L] + (int)(c16 >> (16 - L));
            br->skip(L);
            return (idx >= 0 && idx < 256) ? t->huffval[idx] : -1;
        }
    }
    return -1;
}

PCR_HD int extend(uint32_t v, int s) { return (s && v < (1u << (s - 1))) ? (int)v - (1 << s) + 1 : (int)v; }

// Where a unit's blocks live.  Non-interleaved scans visit only the blocks that cover the
// component's own samples (cw x ch), interleaved scans the MCU-padded grid.
struct UnitGeom {
    uint32_t mcu0, mcu1;        // MCU range [mcu0, mcu1) of the scan handled by this unit
    uint32_t mcu_w;             // MCUs per row of this scan
};

// ---------------------------------------------------------------------------------------
// DC first scan (possibly interleaved).  coef[c]: plane of component c, [bh][bw][64].
// Returns kOk or kEFormat.
// ---------------------------------------------------------------------------------------
PCR_HD int decode_dc_first(BitReader* br, const ImgDesc* img, const ScanDesc* sd, const UnitGeom* ug,
                           const HuffTab* const* tabs, int16_t* const* coef) {
    int pred[kMaxComp] = {0, 0, 0};
    for (uint32_t m = ug->mcu0; m < ug->mcu1; m++) {
        uint32_t my = m / ug->mcu_w, mx = m % ug->mcu_w;
        for (int j = 0; j < sd->ns; j++) {
            int c = sd->comp[j];
            int nx = sd->ns > 1 ? img->hs[c] : 1, ny = sd->ns > 1 ? img->vs[c] : 1;
            for (int by = 0; by < ny; by++) for (int bx = 0; bx < nx; bx++) {
                uint32_t row = sd->ns > 1 ? my * img->vs[c] + by : my, col = sd->ns > 1 ? mx * img->hs[c] + bx : mx;
                br->refill();
                int t = huff_decode(br, tabs[j]);
                if (t < 0 || t > 15) return kEFormat;
                int diff = extend(br->get(t), t);
                pred[j] += diff;
                coef[j][((size_t)row * img->bw[c] + col) * 64] = (int16_t)(pred[j] * (1 << sd->Al));
            }
        }
        if (br->overrun()) return kEFormat;
    }
    return kOk;
}

// DC refinement: one bit per block, OR-ed in at bit Al.
PCR_HD int decode_dc_refine(BitReader* br, const ImgDesc* img, const ScanDesc* sd, const UnitGeom* ug, int16_t* const* coef) {
    for (uint32_t m = ug->mcu0; m < ug->mcu1; m++) {
        uint32_t my = m / ug->mcu_w, mx = m % ug->mcu_w;
        for (int j = 0; j < sd->ns; j++) {
            int c = sd->comp[j];
            int nx = sd->ns > 1 ? img->hs[c] : 1, ny = sd->ns > 1 ? img->vs[c] : 1;
            for (int by = 0; by < ny; by++) for (int bx = 0; bx < nx; bx++) {
                uint32_t row = sd->ns > 1 ? my * img->vs[c] + by : my, col = sd->ns > 1 ? mx * img->hs[c] + bx : mx;
                br->refill();
                if (br->get(1)) coef[j][((size_t)row * img->bw[c] + col) * 64] |= (int16_t)(1 << sd->Al);
            }
        }
        if (br->overrun()) return kEFormat;
    }
    return kOk;
}

// ---------------------------------------------------------------------------------------
// AC first scan of one component, band Ss..Se.  Writes coefficient values (natural order,
// through zz[]) and, per block, the mask of zig-zag positions it made non-zero.
// ---------------------------------------------------------------------------------------
PCR_HD int decode_ac_first(BitReader* br, const ImgDesc* img, const ScanDesc* sd, const UnitGeom* ug, const HuffTab* tab,
                           const uint8_t* zz, int16_t* coef, uint64_t* nzout) {
    int c = sd->comp[0];
    uint32_t eobrun = 0;
    const int Ss = sd->Ss, Se = sd->Se, Al = sd->Al;
    for (uint32_t m = ug->mcu0; m < ug->mcu1; m++) {
        size_t blk = (size_t)(m / ug->mcu_w) * img->bw[c] + (m % ug->mcu_w);
        if (eobrun > 0) { eobrun--; continue; }            // nzout stays 0 (planes are zero-filled)
        uint64_t mask = 0;
        int k = Ss;
        while (k <= Se) {
            br->refill();
            int rs = huff_decode(br, tab);
            if (rs < 0) return kEFormat;
            int r = rs >> 4, s = rs & 15;
            if (s) {
                k += r;
                if (k > Se) return kEFormat;
                int v = extend(br->get(s), s);
                coef[blk * 64 + zz[k]] = (int16_t)(v * (1 << Al));
                mask |= 1ull << k;
                k++;
            } else if (r == 15) k += 16;
            else { eobrun = (1u << r) - 1 + br->get(r); break; }
        }
        nzout[blk] = mask;
        if (br->overrun()) return kEFormat;
    }
    return kOk;
}

// ---------------------------------------------------------------------------------------
// AC refinement scan.  hist planes: masks written by the earlier AC scans of the component.
// Per block this writes
//   nzout  positions that become non-zero in this scan,
//   sign   for those positions, 1 = positive,
//   cbits  the correction bits in reading order (first bit read = bit 0); there is exactly one
//          per already-non-zero coefficient of the band, in zig-zag order.
// ---------------------------------------------------------------------------------------
PCR_HD uint64_t band_mask(int Ss, int Se) { return ((Se >= 63) ? ~0ull : ((1ull << (Se + 1)) - 1)) & ~((1ull << Ss) - 1); }

PCR_HD uint64_t take_correction_bits(BitReader* br, int n) {    // n <= 63; first bit read -> bit 0
    uint64_t out = 0; int done = 0;
    while (n > 0) {
        int t = n > 32 ? 32 : n;
        br->refill();
        uint32_t v = br->get(t);                                // first-read bit is the MSB of the t bits
        uint32_t rv = bitrev32(v) >> (32 - t);
        out |= (uint64_t)rv << done;
        done += t; n -= t;
    }
    return out;
}

PCR_HD int decode_ac_refine(BitReader* br, const ImgDesc* img, const ScanDesc* sd, const UnitGeom* ug, const HuffTab* tab,
                            const uint64_t* const* hist, int nhist, uint64_t* nzout, uint64_t* sign, uint64_t* cbits) {
    int c = sd->comp[0];
    uint32_t eobrun = 0;
    const int Ss = sd->Ss, Se = sd->Se;
    const uint64_t band = band_mask(Ss, Se);
    for (uint32_t m = ug->mcu0; m < ug->mcu1; m++) {
        size_t blk = (size_t)(m / ug->mcu_w) * img->bw[c] + (m % ug->mcu_w);
        uint64_t h = 0;
        for (int q = 0; q < nhist; q++) h |= hist[q][blk];
        h &= band;
        uint64_t newm = 0, sgn = 0, cb = 0; int ncb = 0;
        int k = Ss;
        if (eobrun == 0) {
            while (k <= Se) {
                br->refill();
                int rs = huff_decode(br, tab);
                if (rs < 0) return kEFormat;
                int r = rs >> 4, s = rs & 15;
                uint32_t sbit = 0;
                if (s == 1) sbit = br->get(1);
                else if (s != 0) return kEFormat;
                else if (r < 15) { eobrun = (1u << r) + br->get(r); break; }
                // pass r still-zero positions, then stop on the next still-zero one
                uint64_t from_k = band & ~((1ull << k) - 1);
                uint64_t z = ~h & from_k;
                for (int q = 0; q < r && z; q++) z &= z - 1;
                int pos = z ? __builtin_ctzll(z) : Se + 1;
                if (pos > Se && s == 1) return kEFormat;       // no place left for the new coefficient
                uint64_t upto = (pos >= 64) ? ~0ull : ((1ull << pos) - 1);
                uint64_t cm = h & from_k & upto;
                int n = __builtin_popcountll(cm);
                if (n) { cb |= take_correction_bits(br, n) << ncb; ncb += n; }
                if (s == 1) { newm |= 1ull << pos; sgn |= (uint64_t)sbit << pos; }
                k = pos + 1;
            }
        }
        if (eobrun > 0) {
            uint64_t cm = (k <= Se) ? (h & band & ~((1ull << k) - 1)) : 0;
            int n = __builtin_popcountll(cm);
            if (n) { cb |= take_correction_bits(br, n) << ncb; ncb += n; }
            eobrun--;
        }
        nzout[blk] = newm; sign[blk] = sgn; cbits[blk] = cb;
        if (br->overrun()) return kEFormat;
    }
    return kOk;
}

// ---------------------------------------------------------------------------------------
// Data-parallel part of AC refinement for one coefficient at zig-zag position k of a block.
//   h       mask of positions non-zero before the scan (already restricted to the band)
// ---------------------------------------------------------------------------------------
PCR_HD int16_t refine_apply(int16_t v, int k, uint64_t h, uint64_t newm, uint64_t sgn, uint64_t cb, int Al) {
    uint64_t bit = 1ull << k;
    int p = 1 << Al;
    if (h & bit) {
        int j = __builtin_popcountll(h & (bit - 1));
        if ((cb >> j) & 1) v = (int16_t)(v > 0 ? v + p : v - p);
    } else if (newm & bit) {
        v = (int16_t)((sgn & bit) ? p : -p);
    }
    return v;
}

}  // namespace pcr
