// CPU build of the library's host/device decode functions (pcr_format.h, pcr_entropy.h,
// pcr_pixel.h) driven by plain loops.  Test-only: lets the exact lane code be checked against
// the oracle, with bounds-checked buffers and a debugger, before it runs on a GPU.  The
// kernels' own indexing (k_unstuff, k_pixel tiling) is NOT covered here.
#include <cstdint>
#include <cstring>
#include <vector>
#include "../../paper_1911_00472_amd/csrc/pcr_format.h"
#include "../../paper_1911_00472_amd/csrc/pcr_entropy.h"
#include "../../paper_1911_00472_amd/csrc/pcr_lanes.h"
#include "../../paper_1911_00472_amd/csrc/pcr_pixel.h"

using namespace pcr;

// 0: the AC scans go through the one-wavefront-per-unit decoders (pcr_entropy.h); 1: through the one-lane-per-unit
// decoders (pcr_lanes.h), with what k_refine_history and k_refine_deal do around them done here by plain loops
static int g_lane_decoders = 0;
extern "C" void emul_set_lane_decoders(int on) { g_lane_decoders = on; }

// serial stand-in for the unstuff kernel: same rules (drop stuffed zeros, fill bytes and
// restart markers, stop at any other marker, note interval starts)
static void unstuff(const uint8_t* src, uint32_t L, std::vector<uint8_t>& out, std::vector<uint32_t>& starts) {
    out.clear(); starts.assign(1, 0);
    for (uint32_t q = 0; q < L; q++) {
        uint8_t cur = src[q];
        if (cur != 0xFF) { out.push_back(cur); continue; }
        if (q + 1 >= L) break;
        uint8_t nx = src[q + 1];
        if (nx == 0x00) { out.push_back(0xFF); q++; }
        else if (nx >= 0xD0 && nx <= 0xD7) { starts.push_back((uint32_t)out.size()); q++; }
        else if (nx == 0xFF) continue;
        else break;
    }
}

extern "C" int emul_decode_record(const uint8_t* rec, size_t nbytes, int k, int64_t want_img, int16_t* coef_out, uint8_t* pix_out,
                                  int* W, int* H, int* C) {
    RecordHeader h;
    int rc = parse_record_header(rec, nbytes, &h);
    if (rc) return rc;
    if (k < 1 || k > (int)h.k_avail) return kERange;
    uint32_t n = h.n, G = h.G;
    std::vector<uint32_t> off((size_t)G * n), len((size_t)G * n);
    uint64_t start = h.header_bytes;
    for (uint32_t g = 0; g < h.k_avail; g++) {
        uint64_t pos = start;
        for (uint32_t i = 0; i < n; i++) { uint32_t L = ld_le32(rec + hdr_len_pos(n, G, g, i)); off[(size_t)g * n + i] = (uint32_t)pos; len[(size_t)g * n + i] = L; pos += L; }
        if (h.version == 2) for (uint32_t i = 0; i < n; i++) pos += entry_bytes(ld_le16(rec + hdr_ecount_pos(n, G, g, i)));
        start = pos;
    }
    uint32_t i = (uint32_t)want_img;
    ImgDesc img; std::vector<ScanDesc> sc(G);
    memset(&img, 0, sizeof img);
    parse_image(rec, off.data(), len.data(), n, i, ld_le32(rec + hdr_nscans_pos(n, G, i)), (uint32_t)k, &img, sc.data());
    if (img.status) return img.status;
    *W = img.W; *H = img.H; *C = img.nc;
    size_t poff[4] = {0, 0, 0, 0};
    for (int c = 0; c < img.nc; c++) poff[c + 1] = poff[c] + (size_t)img.bw[c] * img.bh[c] * 64;
    std::vector<int16_t> coef(poff[img.nc], 0);
    std::vector<std::vector<uint64_t>> masks(G);
    uint8_t zz[64]; for (int q = 0; q < 64; q++) zz[q] = (uint8_t)zigzag_natural(q);
    std::vector<std::vector<uint8_t>> cleans(G); std::vector<std::vector<uint32_t>> ivls(G);
    for (uint32_t g = 0; g < img.nscans; g++) {
        const ScanDesc& sd = sc[g];
        std::vector<uint8_t>& clean = cleans[g]; std::vector<uint32_t>& starts = ivls[g];
        clean.reserve(sd.data_len + 64);
        unstuff(rec + sd.data_off, sd.data_len, clean, starts);
        uint32_t nint = sd.ri ? (sd.mcus + sd.ri - 1) / sd.ri : 1;
        if (starts.size() != nint) return kEFormat;
        starts.push_back((uint32_t)clean.size());
        // version 2: the units of a scan without restart markers start at its entry points
        const uint8_t* ent = nullptr; uint32_t stride = kEntryBytes;
        if (h.version == 2 && sd.ri == 0 && !(img.progressive && sd.Ss == 0 && sd.Ah > 0)) {
            const uint32_t field = ld_le16(rec + hdr_ecount_pos(n, G, g, i));
            if (entry_count(field)) {
                uint64_t all = 0, before = 0;
                for (uint32_t q = 0; q < n; q++) { const uint64_t c = entry_bytes(ld_le16(rec + hdr_ecount_pos(n, G, g, q))); all += c; if (q < i) before += c; }
                ent = rec + ld_le64(rec + hdr_group_end_pos(g)) - all + before;
                nint = 1 + entry_count(field); stride = entry_stride(field);
            }
        }
        const uint32_t total_bits = (uint32_t)clean.size() * 8;
        clean.resize((clean.size() + 3) / 4 * 4 + 256, 0xFF);     // look-ahead slack (the lane decoders fetch up to 28 words ahead)
        for (size_t e = 0; e + 3 < clean.size(); e += 4) { std::swap(clean[e], clean[e + 3]); std::swap(clean[e + 1], clean[e + 2]); }   // big-endian words
        int c0 = sd.comp[0];
        size_t plane = (size_t)img.bw[c0] * img.bh[c0];
        if (sd.Ss > 0 && sd.Ah) masks[g].assign(plane * kRefWords, 0);
        if (sd.Ss == 0 && sd.Ah > 0) continue;                     // DC refinement: applied below, in place
        const bool by_lane = g_lane_decoders && sd.Ss > 0 && !is_sequential_scan(sd);
        if (by_lane && sd.Ah) {                                    // (k_refine_history) what is non-zero in the band when the scan starts
            const uint64_t band = band_mask(sd.Ss, sd.Se);
            for (size_t blk = 0; blk < plane; blk++) {
                uint64_t hm = nz_mask_of_block(coef.data() + poff[c0] + blk * 64, sd.Ss, sd.Se);
                for (int q = 0; q < sd.nhist; q++) hm |= masks[sd.hist[q]][kRefNz * plane + blk];
                masks[g][kRefHist * plane + blk] = hm & band;
            }
        }
        for (uint32_t j = 0; j < nint; j++) {
            LaneScan ls;
            ls.mcu_w = sd.mcu_w; ls.mcu0 = sd.ri ? j * sd.ri : 0;
            ls.mcu1 = sd.ri ? (ls.mcu0 + sd.ri < sd.mcus ? ls.mcu0 + sd.ri : sd.mcus) : sd.mcus;
            ls.pred[0] = ls.pred[1] = ls.pred[2] = 0;
            uint32_t byte_off, sub_bits = 0, nbits, pos0 = 0;
            if (ent) {
                const uint8_t* e = ent + (size_t)stride * j;
                uint32_t bit0 = 0, bit1 = total_bits;
                ls.mcu0 = 0; ls.mcu1 = sd.mcus;
                if (j > 0) {
                    ls.mcu0 = ld_le32(e - stride); bit0 = ld_le32(e - stride + 4);
                    if (stride == kEntryBytes) for (int q = 0; q < 3; q++) ls.pred[q] = (int16_t)ld_le16(e - 8 + 2 * q);
                }
                if (j + 1 < nint) { ls.mcu1 = ld_le32(e); bit1 = ld_le32(e + 4); }
                if (!(ls.mcu0 < ls.mcu1 && ls.mcu1 <= sd.mcus && bit0 <= bit1 && bit1 <= total_bits)) return kEFormat;
                byte_off = bit0 >> 3; sub_bits = bit0 & 7; nbits = bit1 - (bit0 & ~7u); pos0 = bit0 & ~7u;
            } else { byte_off = starts[j]; nbits = (starts[j + 1] - starts[j]) * 8; }
            const uint32_t unit_base = ent ? 0u : starts[j];           // what phase 2 of a refinement scan adds to a block's recorded start
            ls.Ss = sd.Ss; ls.Se = sd.Se; ls.Al = sd.Al; ls.ns = sd.ns;
            int16_t* cpl[kMaxComp] = {nullptr, nullptr, nullptr};
            for (int q = 0; q < kMaxComp; q++) {
                int c = q < sd.ns ? sd.comp[q] : 0;
                ls.hs[q] = img.hs[c]; ls.vs[q] = img.vs[c]; ls.bw[q] = img.bw[c]; ls.poff[q] = (uint32_t)poff[c];
                cpl[q] = coef.data() + poff[c];
            }
            if (is_sequential_scan(sd)) {
                std::vector<DcTab> dt(3); std::vector<AcTab> at(3);
                for (int q = 0; q < sd.ns; q++) {
                    dctab_build(&dt[q], rec + sd.dc_off[q]);
                    actab_build(&at[q], rec + sd.ac_offc[q]); actab_pack(&at[q], true, 0, 1);
                }
                SeqTables tb;
                for (int q = 0; q < kMaxComp; q++) { tb.dc[q] = &dt[q]; tb.ac[q] = &at[q]; }
                WindowReader sw;
                sw.init(reinterpret_cast<const uint32_t*>(clean.data()), byte_off, sub_bits, nbits, pos0, tb.ac[0], true, 0, true);
                IndexSink ssink; ssink.init(coef.data(), (uint32_t)coef.size(), 0);
                rc = decode_sequential(&sw, ls, tb, &ssink);
            } else if (sd.Ss == 0 && by_lane && img.progressive && sd.Ah == 0) {
                // the DC first scan with the lane decoder: the unit set up as k_dc_first_lanes sets it up
                static LaneRing ring; static LaneDcTabs dtabs;
                std::vector<int16_t> dense(coef.size() / 64 + 1, 0);
                LaneDcUnit U;
                U.words = reinterpret_cast<const uint32_t*>(clean.data());
                U.bit0 = byte_off * 8 + sub_bits; U.bit1 = byte_off * 8 + nbits;
                U.mcu0 = ls.mcu0; U.mcu1 = ls.mcu1; U.mcu_w = sd.mcu_w; U.ns = (uint32_t)sd.ns; U.Al = (uint32_t)sd.Al;
                const bool one = sd.ns == 1;
                uint32_t hsv[3], vsv[3], bwv[3], pbv[3]; const uint8_t* defv[3];
                for (int q = 0; q < kMaxComp; q++) {
                    const int c = q < sd.ns ? sd.comp[q] : 0;
                    hsv[q] = one ? 1u : img.hs[c]; vsv[q] = one ? 1u : img.vs[c]; bwv[q] = img.bw[c]; pbv[q] = (uint32_t)(poff[c] / 64);
                    defv[q] = rec + sd.dc_off[q < sd.ns ? q : 0];
                }
                U.hs0 = hsv[0]; U.hs1 = hsv[1]; U.hs2 = hsv[2]; U.vs0 = vsv[0]; U.vs1 = vsv[1]; U.vs2 = vsv[2];
                U.bw0 = bwv[0]; U.bw1 = bwv[1]; U.bw2 = bwv[2]; U.pblk0 = pbv[0]; U.pblk1 = pbv[1]; U.pblk2 = pbv[2];
                U.def0 = defv[0]; U.def1 = defv[1]; U.def2 = defv[2];
                U.pred0 = ls.pred[0]; U.pred1 = ls.pred[1]; U.pred2 = ls.pred[2];
                U.dense = dense.data(); U.planes = coef.data(); U.nblocks = (uint32_t)(coef.size() / 64);
                U.ok = true;
                rc = lane_decode_dc_first(U, &ring, &dtabs, 0);
            } else if (sd.Ss == 0) {
                std::vector<DcTab> dt(3);
                for (int q = 0; q < sd.ns; q++) dctab_build(&dt[q], rec + sd.dc_off[q]);
                DcWindowReader dw; dw.init(reinterpret_cast<const uint32_t*>(clean.data()), byte_off, sub_bits, nbits, &dt[0], &dt[1], &dt[2], sd.ns, 0);
                CoefSink dsink; dsink.init(coef.data(), (uint32_t)coef.size(), ls.Al);
                rc = decode_dc_first(&dw, ls, &dsink);
            } else if (by_lane) {
                AcTab at; actab_build(&at, rec + sd.ac_off);
                static LaneRing ring; static LaneHistRing hring;
                LaneUnit U;
                U.words = reinterpret_cast<const uint32_t*>(clean.data());
                U.bit0 = byte_off * 8 + sub_bits; U.bit1 = byte_off * 8 + nbits;
                U.mcu0 = ls.mcu0; U.mcu1 = ls.mcu1; U.mcu_w = sd.mcu_w; U.bw = img.bw[c0];
                U.Ss = sd.Ss; U.Se = sd.Se; U.Al = sd.Al;
                U.plane = cpl[0]; U.plane_elems = (uint32_t)plane * 64;
                U.tab = reinterpret_cast<const LaneTab*>(&at); U.ok = true;
                if (U.mcu0 >= U.mcu1 || U.mcu_w == 0) return kEFormat;
                rc = sd.Ah == 0 ? lane_decode_ac_first(U, &ring, 0) : lane_decode_ac_refine(U, masks[g].data(), (uint32_t)plane, &ring, &hring, 0);
            } else {
                AcTab at; actab_build(&at, rec + sd.ac_off); actab_pack(&at, sd.Ah == 0, 0, 1);
                WindowReader wr; wr.init(reinterpret_cast<const uint32_t*>(clean.data()), byte_off, sub_bits, nbits, pos0, &at, sd.Ah == 0, 0, sd.Ah == 0);
                if (sd.Ah == 0) {
                    IndexSink sink; sink.init(cpl[0], (uint32_t)plane * 64, ls.Al);
                    rc = decode_ac_first(&wr, ls, &sink);
                } else {
                    HistPlanes hp; hp.n = sd.nhist; hp.coef = cpl[0];
                    for (int q = 0; q < kMaxHist; q++) hp.p[q] = sd.nhist ? masks[sd.hist[q < sd.nhist ? q : 0]].data() : nullptr;
                    rc = skim_ac_refine(&wr, ls, hp, masks[g].data(), plane);
                    if (rc) return rc;
                    // phase 2: every block of this interval on its own
                    for (uint32_t mm = ls.mcu0; mm < ls.mcu1; mm++) {
                        size_t blk = (size_t)(mm / sd.mcu_w) * img.bw[c0] + (mm % sd.mcu_w);
                        uint64_t* rec = masks[g].data() + blk;
                        refine_block(reinterpret_cast<const uint32_t*>(clean.data()), unit_base, rec[kRefStart * plane], &at, rec[kRefHist * plane], rec[kRefNz * plane], sd.Ss, sd.Se,
                                     &rec[kRefSign * plane], &rec[kRefPlus * plane]);
                    }
                }
            }
            if (rc) return rc;
        }
        if (by_lane && sd.Ah)                                      // (k_refine_deal) correction bits from reading order to their positions
            for (size_t blk = 0; blk < plane; blk++)
                masks[g][kRefPlus * plane + blk] = deal_bits(masks[g][kRefPlus * plane + blk], masks[g][kRefHist * plane + blk]);
    }
    // refinement, one coefficient at a time (mirrors refine_coefficient of the kernels)
    for (int c = 0; c < img.nc; c++) {
        size_t plane = (size_t)img.bw[c] * img.bh[c];
        for (uint32_t row = 0; row < img.bh[c]; row++) for (uint32_t col = 0; col < img.bw[c]; col++) for (int kk = 0; kk < 64; kk++) {
            size_t blk = (size_t)row * img.bw[c] + col;
            bool covered = row < img.ch[c] && col < img.cw[c];
            int16_t* cp = coef.data() + poff[c] + blk * 64 + kk;     // internal order: element k = zig-zag position k
            int16_t v = *cp;
            for (uint32_t g = 0; g < img.nscans; g++) {
                const ScanDesc& sd = sc[g];
                if (sd.Ss == 0) {
                    if (kk != 0 || sd.Ah == 0) continue;
                    int j = -1; uint32_t before = 0, bpm = 0;
                    for (int q = 0; q < sd.ns; q++) { int cq = sd.comp[q]; uint32_t nb = sd.ns > 1 ? (uint32_t)img.hs[cq] * img.vs[cq] : 1; if (cq == c) { j = q; before = bpm; } bpm += nb; }
                    if (j < 0) continue;
                    uint32_t m, within;
                    if (sd.ns > 1) { m = (row / img.vs[c]) * sd.mcu_w + col / img.hs[c]; within = before + (row % img.vs[c]) * img.hs[c] + col % img.hs[c]; }
                    else { if (!covered) continue; m = row * sd.mcu_w + col; within = 0; }
                    uint32_t ivl = sd.ri ? m / sd.ri : 0, bit = (m - ivl * sd.ri) * bpm + within;
                    if (bit >= (ivls[g][ivl + 1] - ivls[g][ivl]) * 8) return kEFormat;
                    if (dc_refine_bit(reinterpret_cast<const uint32_t*>(cleans[g].data()), ivls[g][ivl], bit)) v |= (int16_t)(1 << sd.Al);
                } else if (kk != 0 && covered && sd.comp[0] == c && sd.Ah != 0 && kk >= sd.Ss && kk <= sd.Se) {
                    const uint64_t* mk = masks[g].data();
                    const uint64_t* rec = mk + blk;
                    v = refine_apply(v, kk, rec[kRefNz * plane], rec[kRefSign * plane], rec[kRefPlus * plane], sd.Al);
                }
            }
            *cp = v;
        }
    }
    {   // internal (zig-zag inside each block) -> natural order
        std::vector<int16_t> nat(coef.size());
        for (size_t e = 0; e < coef.size(); e++) nat[(e & ~(size_t)63) + zz[e & 63]] = coef[e];
        coef.swap(nat);
    }
    if (coef_out) memcpy(coef_out, coef.data(), coef.size() * sizeof(int16_t));
    if (pix_out) {
        std::vector<std::vector<float>> pl(img.nc);
        for (int c = 0; c < img.nc; c++) {
            uint32_t pw = img.bw[c] * 8;
            pl[c].assign((size_t)pw * img.bh[c] * 8, 0.f);
            float qn[64];
            const uint8_t* q = rec + img.qoff[img.tq[c]];
            for (int kk = 0; kk < 64; kk++) qn[zz[kk]] = img.qprec[img.tq[c]] ? (float)ld_be16(q + 2 * kk) : (float)q[kk];
            for (uint32_t by = 0; by < img.bh[c]; by++) for (uint32_t bx = 0; bx < img.bw[c]; bx++) {
                const int16_t* blk = coef.data() + poff[c] + ((size_t)by * img.bw[c] + bx) * 64;
                float t[64];
                for (int v = 0; v < 8; v++) { float in[8], res[8]; for (int u = 0; u < 8; u++) in[u] = (float)blk[v * 8 + u] * qn[v * 8 + u]; idct8(in, res); for (int x = 0; x < 8; x++) t[v * 8 + x] = res[x]; }
                for (int x = 0; x < 8; x++) { float in[8], res[8]; for (int v = 0; v < 8; v++) in[v] = t[v * 8 + x]; idct8(in, res);
                    for (int y = 0; y < 8; y++) pl[c][(size_t)(by * 8 + y) * pw + bx * 8 + x] = clamp255(res[y] + 128.f); }
            }
        }
        for (uint32_t y = 0; y < img.H; y++) for (uint32_t x = 0; x < img.W; x++) {
            float s[3];
            for (int c = 0; c < img.nc; c++) s[c] = pl[c][(size_t)(y * img.vs[c] / img.vmax) * (img.bw[c] * 8) + x * img.hs[c] / img.hmax];
            uint8_t* o = pix_out + ((size_t)y * img.W + x) * img.nc;
            if (img.nc == 1) o[0] = round_u8(s[0]); else ycc_to_rgb(s[0], s[1], s[2], o);
        }
    }
    return kOk;
}
