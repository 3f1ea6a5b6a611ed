// Record header and JPEG marker parsing, compiled for host and device.
//
// Record layout (paper Section 3, record figure: metadata first, then the scan groups in
// order of fidelity; raw struct serialisation, Section 5 "Loader"), little endian:
//   "PCR1" | u32 version | u32 n | u32 G | u64 header_bytes | u64 group_end[G] | i32 label[n]
//   | u32 n_scans[n] | u32 len[G][n] | padding | group 1 | group 2 | ...
// Group g holds the g-th scan region of every image back to back.  A region is the slice of
// the image's progressive JPEG file between the ends of two consecutive scans (Section 5,
// "Encoding"): region 1 starts with SOI and carries the frame header and tables, every
// later region carries the tables and the SOS header of its one scan followed by the
// entropy-coded data.
//
// Version 2 adds entry points, an index INTO the scans (the paper's metadata only says where each scan group
// starts; Section 4.2 names the decode of a scan as the bottleneck, and a scan of a stock file is one serial
// stream): after len[G][n] the header carries
//   u32 entry_interval | u32 0 | u16 ecount[G][n]
// and group g ends with the entries of its scans, image after image, ecount[g][i] entries of 16 bytes each:
//   u32 mcu | u32 bit | i16 pred[3] | u16 0
// "decoding of this scan may start at MCU `mcu` of the scan (block `mcu` of a scan of one component), at bit `bit`
// of its entropy-coded data counted without the stuffed zero bytes, with the DC predictions `pred` of the scan's
// components (scans that code DC differences), and no end-of-band run is pending there".  Entries are in
// increasing order; scans with restart markers and DC refinement scans have none.  The image bytes are exactly
// those of version 1: region lengths and offsets do not change, group_end[g] includes the group's entries.
#pragma once
#include "pcr_common.h"

namespace pcr {

struct RecordHeader {
    uint32_t n, G;
    uint64_t header_bytes;
    uint32_t k_avail;                      // scan groups wholly inside the bytes given
    uint32_t version;                      // 1, or 2: with entry points
    uint32_t entry_interval;               // version 2: MCUs between entry points the writer aimed at (informative)
};
// Version 2: an entry point is 16 bytes (MCU, bit offset, three DC predictions, two reserved bytes), or 8 (MCU and bit
// offset only) where the scan has no DC predictions to resume -- the AC scans, nearly all entries of a record.  The
// header's 16-bit entry count of an (image, scan) carries the form in its top bit.
constexpr uint32_t kEntryBytes = 16, kEntryBytesShort = 8, kEntryShortFlag = 0x8000u, kMaxEntriesPerScan = 0x7FFFu;

PCR_HD uint64_t hdr_group_end_pos(uint32_t g) { return 24 + 8ull * g; }
PCR_HD uint64_t hdr_label_pos(uint32_t G, uint32_t i) { return 24 + 8ull * G + 4ull * i; }
PCR_HD uint64_t hdr_nscans_pos(uint32_t n, uint32_t G, uint32_t i) { return 24 + 8ull * G + 4ull * n + 4ull * i; }
PCR_HD uint64_t hdr_len_pos(uint32_t n, uint32_t G, uint32_t g, uint32_t i) { return 24 + 8ull * G + 8ull * n + 4ull * ((uint64_t)g * n + i); }
PCR_HD uint64_t hdr_entry_interval_pos(uint32_t n, uint32_t G) { return hdr_len_pos(n, G, G, 0); }                  // version 2
PCR_HD uint64_t hdr_ecount_pos(uint32_t n, uint32_t G, uint32_t g, uint32_t i) { return hdr_len_pos(n, G, G, 0) + 8 + 2ull * ((uint64_t)g * n + i); }
PCR_HD uint32_t ld_le16(const uint8_t* p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8); }
// the entry-count field of the header taken apart
PCR_HD uint32_t entry_count(uint32_t field) { return field & kMaxEntriesPerScan; }
PCR_HD uint32_t entry_stride(uint32_t field) { return (field & kEntryShortFlag) ? kEntryBytesShort : kEntryBytes; }
PCR_HD uint64_t entry_bytes(uint32_t field) { return (uint64_t)entry_count(field) * entry_stride(field); }

// Validate the fixed part of the header.  `bytes` must hold at least min(nbytes, header).
PCR_HD int parse_record_header(const uint8_t* bytes, uint64_t nbytes, RecordHeader* h) {
    if (nbytes < 24) return kETruncated;
    if (bytes[0] != 'P' || bytes[1] != 'C' || bytes[2] != 'R' || bytes[3] != '1') return kEFormat;
    h->version = ld_le32(bytes + 4);
    if (h->version != 1 && h->version != 2) return kEUnsupported;
    h->n = ld_le32(bytes + 8); h->G = ld_le32(bytes + 12); h->header_bytes = ld_le64(bytes + 16);
    if (h->n == 0 || h->G == 0 || h->G > 64 || h->n > (1u << 24)) return kEFormat;
    uint64_t need = h->version == 2 ? hdr_ecount_pos(h->n, h->G, h->G, 0) : hdr_len_pos(h->n, h->G, h->G, 0);
    if (h->header_bytes < need) return kEFormat;
    if (nbytes < h->header_bytes) return kETruncated;
    h->entry_interval = h->version == 2 ? ld_le32(bytes + hdr_entry_interval_pos(h->n, h->G)) : 0;
    uint64_t prev = h->header_bytes; uint32_t k = 0;
    for (uint32_t g = 0; g < h->G; g++) {
        uint64_t e = ld_le64(bytes + hdr_group_end_pos(g));
        if (e < prev) return kEFormat;
        if (e <= nbytes && k == g) k = g + 1;
        prev = e;
    }
    h->k_avail = k;
    return kOk;
}

// ---------------------------------------------------------------------------------------
// Marker parsing of one image: walks the headers of regions 0..kmax-1 (never the
// entropy-coded data) and fills the image and scan descriptors.
//   rec      record bytes (host or device pointer, matching where this runs)
//   off,len  index tables [G][n] (absolute offsets / lengths of the regions)
// Every read is bounds-checked against the region it belongs to.
// ---------------------------------------------------------------------------------------
struct ParseState {
    uint32_t dht[2][4];                    // offset of BITS of the table last defined for (class, id)
    uint16_t ri;
    int have_frame;
};

PCR_HD void setup_geometry(ImgDesc* d) {
    d->hmax = 1; d->vmax = 1;
    for (int c = 0; c < d->nc; c++) { if (d->hs[c] > d->hmax) d->hmax = d->hs[c]; if (d->vs[c] > d->vmax) d->vmax = d->vs[c]; }
    d->mcux = (uint16_t)((d->W + 8 * d->hmax - 1) / (8 * d->hmax));
    d->mcuy = (uint16_t)((d->H + 8 * d->vmax - 1) / (8 * d->vmax));
    for (int c = 0; c < d->nc; c++) {
        d->bw[c] = (uint16_t)(d->mcux * d->hs[c]); d->bh[c] = (uint16_t)(d->mcuy * d->vs[c]);
        uint32_t xc = ((uint32_t)d->W * d->hs[c] + d->hmax - 1) / d->hmax, yc = ((uint32_t)d->H * d->vs[c] + d->vmax - 1) / d->vmax;
        d->cw[c] = (uint16_t)((xc + 7) / 8); d->ch[c] = (uint16_t)((yc + 7) / 8);
    }
}

PCR_HD int parse_region(const uint8_t* rec, uint32_t p, uint32_t end, int first_region, ParseState* st, ImgDesc* img,
                        ScanDesc* scans, uint32_t g) {
    ScanDesc* sd = &scans[g];
    if (first_region) {
        if (end - p < 2 || rec[p] != 0xFF || rec[p + 1] != 0xD8) return kEFormat;
        p += 2;
    }
    while (true) {
        if (end - p < 4) return kEFormat;
        if (rec[p] != 0xFF) return kEFormat;
        uint32_t m = rec[p + 1];
        if (m == 0xFF) { p++; continue; }
        uint32_t L = ld_be16(rec + p + 2);
        if (L < 2 || L + 2 > end - p) return kEFormat;
        uint32_t s = p + 4, se = p + 2 + L;
        p = se;
        if (m == 0xDB) {
            while (s < se) {
                uint32_t pq = rec[s] >> 4, tq = rec[s] & 15; s++;
                if (tq > 3 || pq > 1 || se - s < 64 * (pq + 1)) return kEFormat;
                img->qoff[tq] = s; img->qprec[tq] = (uint8_t)pq;
                s += 64 * (pq + 1);
            }
        } else if (m == 0xC0 || m == 0xC1 || m == 0xC2) {
            if (st->have_frame || se - s < 6) return kEFormat;
            if (rec[s] != 8) return kEUnsupported;
            img->progressive = (m == 0xC2);
            img->H = (uint16_t)ld_be16(rec + s + 1); img->W = (uint16_t)ld_be16(rec + s + 3); img->nc = rec[s + 5];
            if (img->H == 0 || img->W == 0) return kEUnsupported;
            if (img->nc != 1 && img->nc != 3) return kEUnsupported;
            if (se - s < 6u + 3u * img->nc) return kEFormat;
            for (int c = 0; c < img->nc; c++) {
                img->cid[c] = rec[s + 6 + 3 * c]; img->hs[c] = rec[s + 7 + 3 * c] >> 4; img->vs[c] = rec[s + 7 + 3 * c] & 15; img->tq[c] = rec[s + 8 + 3 * c];
                if (img->hs[c] < 1 || img->hs[c] > 2 || img->vs[c] < 1 || img->vs[c] > 2 || img->tq[c] > 3) return kEUnsupported;
            }
            if (img->nc == 1) { img->hs[0] = 1; img->vs[0] = 1; }
            setup_geometry(img);
            st->have_frame = 1;
        } else if ((m >= 0xC3 && m <= 0xCF && m != 0xC4 && m != 0xC8 && m != 0xCC) || m == 0xDC) {
            return kEUnsupported;                  // lossless, hierarchical, arithmetic coding, DNL
        } else if (m == 0xC4) {
            while (s < se) {
                uint32_t tc = rec[s] >> 4, th = rec[s] & 15;
                if (tc > 1 || th > 3 || se - s < 17) return kEFormat;
                uint32_t nv = 0; for (int i = 0; i < 16; i++) nv += rec[s + 1 + i];
                if (nv > 256 || se - s < 17 + nv) return kEFormat;
                st->dht[tc][th] = s + 1;
                s += 17 + nv;
            }
        } else if (m == 0xDD) {
            if (se - s < 2) return kEFormat;
            st->ri = (uint16_t)ld_be16(rec + s);
        } else if (m == 0xDA) {
            if (!st->have_frame || se - s < 1) return kEFormat;
            uint32_t ns = rec[s];
            if (ns < 1 || ns > img->nc || se - s < 1 + 2 * ns + 3) return kEFormat;
            sd->ns = (uint8_t)ns;
            uint32_t td[kMaxComp], ta[kMaxComp];
            for (uint32_t j = 0; j < ns; j++) {
                int c = -1;
                for (int q = 0; q < img->nc; q++) if (img->cid[q] == rec[s + 1 + 2 * j]) c = q;
                if (c < 0) return kEFormat;
                sd->comp[j] = (uint8_t)c; td[j] = rec[s + 2 + 2 * j] >> 4; ta[j] = rec[s + 2 + 2 * j] & 15;
                if (td[j] > 3 || ta[j] > 3) return kEFormat;
            }
            sd->Ss = rec[s + 1 + 2 * ns]; sd->Se = rec[s + 2 + 2 * ns]; sd->Ah = rec[s + 3 + 2 * ns] >> 4; sd->Al = rec[s + 3 + 2 * ns] & 15;
            for (int j = 0; j < kMaxComp; j++) sd->ac_offc[j] = 0;
            if (!img->progressive) {
                // Sequential (baseline) file, the format a record of non-progressive images holds (one scan group, or
                // one per component): the scan header must say "all 64 coefficients, full precision".
                if (sd->Ss != 0 || sd->Se != 63 || sd->Ah != 0 || sd->Al != 0) return kEFormat;
                for (uint32_t j = 0; j < ns; j++) {
                    if (!st->dht[0][td[j]] || !st->dht[1][ta[j]]) return kEFormat;
                    sd->dc_off[j] = st->dht[0][td[j]]; sd->ac_offc[j] = st->dht[1][ta[j]];
                }
                sd->ac_off = sd->ac_offc[0];
            } else {
                if (sd->Ss > sd->Se || sd->Se > 63 || (sd->Ss == 0 && sd->Se != 0) || (sd->Ss > 0 && ns != 1) || sd->Al > 13) return kEFormat;
                if (sd->Ah != 0 && sd->Ah != sd->Al + 1) return kEFormat;
                for (uint32_t j = 0; j < ns; j++) {
                    sd->dc_off[j] = 0;
                    if (sd->Ss == 0 && sd->Ah == 0) { if (!st->dht[0][td[j]]) return kEFormat; sd->dc_off[j] = st->dht[0][td[j]]; }
                }
                sd->ac_off = 0;
                if (sd->Ss > 0) { if (!st->dht[1][ta[0]]) return kEFormat; sd->ac_off = st->dht[1][ta[0]]; }
            }
            sd->ri = st->ri;
            if (ns > 1) { sd->mcu_w = img->mcux; sd->mcus = (uint32_t)img->mcux * img->mcuy; }
            else { sd->mcu_w = img->cw[sd->comp[0]]; sd->mcus = (uint32_t)img->cw[sd->comp[0]] * img->ch[sd->comp[0]]; }
            sd->data_off = p; sd->data_len = end - p;
            // A refinement scan works on the positions of its band that are already non-zero.  Those made
            // non-zero by AC first scans are read back from the coefficients; those added by earlier
            // refinement scans of the component (not applied to the coefficients yet) come from the masks
            // those scans leave, so they are listed here.
            sd->nhist = 0;
            if (sd->Ss > 0) {
                bool has_first = false;
                for (uint32_t q = 0; q < g; q++) {
                    const ScanDesc* e = &scans[q];
                    if (e->Ss > 0 && e->comp[0] == sd->comp[0] && e->Ss <= sd->Se && sd->Ss <= e->Se) {
                        if (e->Ah == 0) { has_first = true; continue; }
                        if (sd->nhist >= kMaxHist) return kEUnsupported;
                        sd->hist[sd->nhist++] = (uint8_t)q;
                    }
                }
                if (sd->Ah > 0 && !has_first) return kEFormat;
                if (sd->Ah == 0) sd->nhist = 0;            // first scans need no history
            }
            sd->valid = 1;
            return kOk;
        }
        // APPn, COM, anything else with a length: skipped
    }
}

// Parse image i: regions 0..kmax-1.  scans points at this image's G descriptors.
PCR_HD void parse_image(const uint8_t* rec, const uint32_t* off, const uint32_t* len, uint32_t n, uint32_t i,
                        uint32_t nscans_i, uint32_t kmax, ImgDesc* img, ScanDesc* scans) {
    ParseState st;
    for (int a = 0; a < 2; a++) for (int b = 0; b < 4; b++) st.dht[a][b] = 0;
    st.ri = 0; st.have_frame = 0;
    for (int t = 0; t < 4; t++) { img->qoff[t] = 0; img->qprec[t] = 0; }
    img->status = kOk; img->nscans = 0; img->nc = 0; img->W = 0; img->H = 0;
    for (int c = 0; c < kMaxComp; c++) img->zmax[c] = 0;
    img->pad = 0;
    uint32_t upto = nscans_i < kmax ? nscans_i : kmax;
    for (uint32_t g = 0; g < upto; g++) {
        scans[g].valid = 0;
        uint32_t p = off[(size_t)g * n + i], L = len[(size_t)g * n + i];
        int rc = parse_region(rec, p, p + L, g == 0, &st, img, scans, g);
        if (rc != kOk) { img->status = rc; return; }
        img->nscans = g + 1;
        for (int j = 0; j < scans[g].ns; j++) {
            const int c = scans[g].comp[j];
            if (scans[g].Se + 1 > img->zmax[c]) img->zmax[c] = (uint8_t)(scans[g].Se + 1);
        }
    }
    if (img->nscans == 0) { img->status = kEFormat; return; }
    // the refinement scans of a component are replayed from a list of fixed length when its coefficients are loaded
    for (int c = 0; c < img->nc; c++) {
        int nref = 0;
        for (uint32_t g = 0; g < img->nscans; g++) {
            if (scans[g].Ah == 0) continue;
            for (int j = 0; j < scans[g].ns; j++) if (scans[g].comp[j] == c) nref++;
        }
        if (nref > kApplyMaxScans) { img->status = kEUnsupported; return; }
    }
    for (int c = 0; c < img->nc; c++) if (!img->qoff[img->tq[c]]) { img->status = kEFormat; return; }
}

}  // namespace pcr
