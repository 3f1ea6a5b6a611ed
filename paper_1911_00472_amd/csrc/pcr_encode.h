// Host side of record creation (paper Section 5, "Encoding"): find where each scan of a JPEG file ends,
// group the scans of many files into one record with its index in front, and re-code the quantised
// coefficients of a file as a progressive file (the lossless transcode the paper does with a stock tool
// before it groups scans: same coefficients, ten scans for colour, six for gray).
//
// Everything here runs on the CPU: it is done once per dataset, not per batch.  The coefficients a transcode
// starts from come from the device decoder (pcr_decode_coefficients), which reads baseline and progressive
// sources alike.
#pragma once
#include <algorithm>
#include <atomic>
#include <cstring>
#include <thread>
#include <vector>

#include "pcr_format.h"
#include "pcr_entropy.h"
#include "pcr_hist.h"

namespace pcr {
namespace enc {

// ---- scan splitter --------------------------------------------------------------------------------------
// Region s of a file ends where the entropy-coded data of its scan s ends: at the first 0xFF that is not
// followed by 0x00 (a stuffed byte), by a restart marker or by more 0xFF fill leading up to one of those.
// The last region runs to the end of the file.  Returns the number of scans (0: not a well-formed file, or
// more than max_ends scans).
inline int scan_ends(const uint8_t* d, size_t n, uint64_t* ends, int max_ends) {
    if (n < 4 || d[0] != 0xFF || d[1] != 0xD8) return 0;
    int count = 0;
    size_t p = 2;
    auto is_data_follow = [](uint8_t x) { return x == 0x00 || (x >= 0xD0 && x <= 0xD7); };
    while (p + 4 <= n) {
        if (d[p] != 0xFF) return 0;
        const uint8_t m = d[p + 1];
        if (m == 0xFF) { p++; continue; }                      // fill before a marker
        if (m == 0xD9) break;
        const size_t len = ((size_t)d[p + 2] << 8) | d[p + 3];
        if (len < 2 || p + 2 + len > n) return 0;
        p += 2 + len;
        if (m != 0xDA) continue;
        // entropy-coded data: hop from 0xFF to 0xFF
        for (;;) {
            const void* hit = p < n ? memchr(d + p, 0xFF, n - p) : nullptr;
            if (!hit) return 0;                                // data runs off the file: no EOI
            p = (size_t)((const uint8_t*)hit - d);
            size_t q = p + 1;
            while (q < n && d[q] == 0xFF) q++;                 // a run of 0xFF counts as one
            if (q >= n) return 0;
            if (is_data_follow(d[q])) { p = q + 1; continue; }
            break;                                             // a real marker: the region ends at the first 0xFF of the run
        }
        if (count >= max_ends) return 0;
        ends[count++] = p;
    }
    if (count == 0) return 0;
    ends[count - 1] = n;
    return count;
}

// ---- record writer --------------------------------------------------------------------------------------
struct RecordPlan {
    uint32_t n = 0, G = 0;
    uint64_t header_bytes = 0, total = 0;
    std::vector<uint32_t> nscans;                              // [n]
    std::vector<uint64_t> ends;                                // [n][64] region ends of every file
};

constexpr int kMaxScansPerFile = 64;

inline int plan_record(const void* const* files, const size_t* sizes, uint32_t n, RecordPlan* P) {
    if (n == 0 || n > (1u << 24)) return kERange;
    P->n = n; P->G = 0; P->nscans.assign(n, 0); P->ends.assign((size_t)n * kMaxScansPerFile, 0);
    uint64_t payload = 0;
    for (uint32_t i = 0; i < n; i++) {
        if (!files[i]) return kEArg;
        const int s = scan_ends((const uint8_t*)files[i], sizes[i], &P->ends[(size_t)i * kMaxScansPerFile], kMaxScansPerFile);
        if (s <= 0) return kEFormat;
        P->nscans[i] = (uint32_t)s;
        if ((uint32_t)s > P->G) P->G = (uint32_t)s;
        payload += sizes[i];
    }
    const uint64_t raw = hdr_len_pos(n, P->G, P->G, 0);
    P->header_bytes = (raw + 63) / 64 * 64;
    P->total = P->header_bytes + payload;
    if (P->total >= (1ull << 32)) return kEUnsupported;        // offsets inside a record are 32 bits
    return kOk;
}

inline void st_le32(uint8_t* p, uint32_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24); }
inline void st_le64(uint8_t* p, uint64_t v) { st_le32(p, (uint32_t)v); st_le32(p + 4, (uint32_t)(v >> 32)); }

inline void write_record(const RecordPlan& P, const void* const* files, const int32_t* labels, uint8_t* out) {
    const uint32_t n = P.n, G = P.G;
    memset(out, 0, P.header_bytes);
    memcpy(out, "PCR1", 4);
    st_le32(out + 4, 1); st_le32(out + 8, n); st_le32(out + 12, G); st_le64(out + 16, P.header_bytes);
    uint64_t pos = P.header_bytes;
    for (uint32_t g = 0; g < G; g++) {
        for (uint32_t i = 0; i < n; i++) {
            uint32_t len = 0;
            if (g < P.nscans[i]) {
                const uint64_t* e = &P.ends[(size_t)i * kMaxScansPerFile];
                const uint64_t from = g ? e[g - 1] : 0;
                len = (uint32_t)(e[g] - from);
                memcpy(out + pos, (const uint8_t*)files[i] + from, len);
                pos += len;
            }
            st_le32(out + hdr_len_pos(n, G, g, i), len);
        }
        st_le64(out + hdr_group_end_pos(g), pos);
    }
    for (uint32_t i = 0; i < n; i++) {
        st_le32(out + hdr_label_pos(G, i), labels ? (uint32_t)labels[i] : 0u);
        st_le32(out + hdr_nscans_pos(n, G, i), P.nscans[i]);
    }
}

// ---- entry points (record version 2) ----------------------------------------------------------------------
// A scan of a stock file is one serial stream.  The record writer walks every scan once and notes, about every
// `interval` MCUs, a place where a decoder may start: a block boundary outside any end-of-band run, the bit
// offset of that place in the scan's data without the stuffed bytes, and the DC predictions there.  The walk
// needs no coefficient values, only which positions of every block are non-zero so far (the refinement scans'
// zero runs skip those).  Scans with restart markers need no entries: every restart interval is a start already.
struct EntryPoint { uint32_t mcu, bit; int16_t pred[3]; uint16_t zero; };
static_assert(sizeof(EntryPoint) == kEntryBytes, "entry layout");

struct BitCursor {
    const uint8_t* d; uint64_t nbits, pos; bool bad;
    // the 32 bits at the cursor (the buffer is padded beyond its end)
    uint32_t peek() const {
        const uint8_t* p = d + (pos >> 3);
        const uint64_t v = ((uint64_t)p[0] << 32) | ((uint64_t)p[1] << 24) | ((uint64_t)p[2] << 16) | ((uint64_t)p[3] << 8) | p[4];
        return (uint32_t)(v >> (8 - (pos & 7)));
    }
    void skip(uint32_t n) { pos += n; if (pos > nbits) bad = true; }
    uint32_t take(uint32_t n) { const uint32_t v = n ? peek() >> (32 - n) : 0; skip(n); return v; }
};

// Entropy-coded data of a scan without stuffed zeros, fill bytes and restart markers; starts[j] = first byte of
// restart interval j.  Stops at the first other marker.
inline void unstuff_scan(const uint8_t* src, uint32_t L, std::vector<uint8_t>* out, std::vector<uint32_t>* starts) {
    out->clear(); starts->assign(1, 0);
    for (uint32_t q = 0; q < L; q++) {
        const uint8_t cur = src[q];
        if (cur != 0xFF) { out->push_back(cur); continue; }
        if (q + 1 >= L) break;
        const uint8_t nx = src[q + 1];
        if (nx == 0x00) { out->push_back(0xFF); q++; }
        else if (nx >= 0xD0 && nx <= 0xD7) { starts->push_back((uint32_t)out->size()); q++; }
        else if (nx == 0xFF) continue;
        else break;
    }
}

// ent[g]: entry points of scan g of the file (empty where there are none, also for every scan from the first one
// this walk cannot follow).  ends: the file's region ends (scan_ends).  Returns kOk, or why the frame was refused.
inline int find_entry_points(const uint8_t* file, const uint64_t* ends, uint32_t nscans, uint32_t interval, std::vector<EntryPoint>* ent) {
    for (uint32_t g = 0; g < nscans; g++) ent[g].clear();
    if (interval == 0 || nscans > (uint32_t)kMaxScansPerFile) return kOk;
    uint32_t off[kMaxScansPerFile], len[kMaxScansPerFile];
    for (uint32_t g = 0; g < nscans; g++) { off[g] = g ? (uint32_t)ends[g - 1] : 0u; len[g] = (uint32_t)ends[g] - off[g]; }
    ImgDesc img; std::vector<ScanDesc> sc(nscans);
    memset(&img, 0, sizeof img); memset(sc.data(), 0, sizeof(ScanDesc) * nscans);
    parse_image(file, off, len, 1, 0, nscans, nscans, &img, sc.data());
    if (img.status != kOk) return img.status;
    std::vector<uint64_t> nz[kMaxComp];
    for (int c = 0; c < img.nc; c++) nz[c].assign((size_t)img.bw[c] * img.bh[c], 0);
    std::vector<uint8_t> clean; std::vector<uint32_t> starts;
    std::vector<DcTab> dt(kMaxComp); std::vector<AcTab> at(kMaxComp);
    for (uint32_t g = 0; g < nscans; g++) {
        const ScanDesc& sd = sc[g];
        const bool seq = !img.progressive;
        if (!seq && sd.Ss == 0 && sd.Ah > 0) continue;               // DC refinement: one bit per block, nothing to walk
        unstuff_scan(file + sd.data_off, sd.data_len, &clean, &starts);
        const uint32_t nint = sd.ri ? (sd.mcus + sd.ri - 1) / sd.ri : 1;
        if (starts.size() != nint) return kOk;                        // damaged: the decoder will say so
        starts.push_back((uint32_t)clean.size());
        const uint64_t total_bits = (uint64_t)clean.size() * 8;
        clean.resize(clean.size() + 16, 0xFF);
        if (seq || sd.Ss == 0) for (int j = 0; j < sd.ns; j++) dctab_build(&dt[j], file + sd.dc_off[j]);
        if (seq) for (int j = 0; j < sd.ns; j++) actab_build(&at[j], file + sd.ac_offc[j]);
        else if (sd.Ss > 0) actab_build(&at[0], file + sd.ac_off);
        const int c0 = sd.comp[0];
        const uint64_t band = (sd.Se >= 63 ? ~0ull : ((1ull << (sd.Se + 1)) - 1)) & ~((1ull << sd.Ss) - 1);
        std::vector<EntryPoint>& E = ent[g];
        BitCursor b{clean.data(), total_bits, 0, false};
        for (uint32_t iv = 0; iv < nint && !b.bad; iv++) {
            b.pos = (uint64_t)starts[iv] * 8;
            b.nbits = (uint64_t)starts[iv + 1] * 8;
            int pred[kMaxComp] = {0, 0, 0};
            uint32_t eobrun = 0;
            const uint32_t m0 = sd.ri ? iv * sd.ri : 0, m1 = sd.ri ? std::min(m0 + sd.ri, sd.mcus) : sd.mcus;
            // AC refinement scans get an entry every interval / 2: a symbol of theirs takes a decoder more than twice as
            // long as one of an AC first scan (zero runs are counted against the block's history, correction bits follow),
            // and a launch of the lane-per-unit decoders takes as long as its longest unit.  So do DC first scans: an MCU
            // of theirs is several symbols (six with 4:2:0 sampling), each found by comparing with the table's codes.
            const bool halved = !seq && interval >= 2 && ((sd.Ss > 0 && sd.Ah > 0) || sd.Ss == 0);
            const uint32_t step = halved ? interval / 2 : interval;
            uint32_t next_entry = step;
            for (uint32_t m = m0; m < m1 && !b.bad; m++) {
                if (sd.ri == 0 && m >= next_entry && eobrun == 0 && E.size() < kMaxEntriesPerScan) {
                    EntryPoint e; e.mcu = m; e.bit = (uint32_t)b.pos; e.zero = (!seq && sd.Ss > 0) ? 1 : 0;   // (in memory: 1 = written in the short form)
                    for (int j = 0; j < kMaxComp; j++) e.pred[j] = (int16_t)pred[j];
                    E.push_back(e);
                    next_entry = (m / step + 1) * step;
                }
                if (seq || sd.Ss == 0) {                             // blocks of every scan component of the MCU
                    for (int j = 0; j < sd.ns && !b.bad; j++) {
                        const int c = sd.comp[j];
                        const uint32_t nb = sd.ns > 1 ? (uint32_t)img.hs[c] * img.vs[c] : 1u;
                        for (uint32_t q = 0; q < nb && !b.bad; q++) {
                            const uint32_t e = dc_code(&dt[j], b.peek());
                            if (!e) { b.bad = true; break; }
                            b.skip(e >> 4);
                            pred[j] += extend(b.take(e & 15), (int)(e & 15));
                            if (!seq) continue;
                            for (int k = 1; k < 64 && !b.bad;) {
                                const uint32_t a = ac_code(&at[j], b.peek());
                                if (!a) { b.bad = true; break; }
                                const uint32_t r = (a >> 4) & 15, sz = a & 15;
                                b.skip(a >> 8);
                                if (sz) { k += (int)r + 1; b.skip(sz); }
                                else if (r == 15) k += 16;
                                else break;
                            }
                        }
                    }
                    continue;
                }
                uint64_t& h = nz[c0][(size_t)(m / sd.mcu_w) * img.bw[c0] + m % sd.mcu_w];
                if (sd.Ah == 0) {                                    // AC first
                    if (eobrun) { eobrun--; continue; }
                    for (int k = sd.Ss; k <= sd.Se && !b.bad;) {
                        const uint32_t a = ac_code(&at[0], b.peek());
                        if (!a) { b.bad = true; break; }
                        const uint32_t r = (a >> 4) & 15, sz = a & 15;
                        b.skip(a >> 8);
                        if (sz) {
                            k += (int)r;
                            if (k > sd.Se) { b.bad = true; break; }
                            b.skip(sz); h |= 1ull << k; k++;
                        } else if (r == 15) k += 16;
                        else { eobrun = (1u << r) - 1 + b.take(r); break; }
                    }
                } else {                                             // AC refinement
                    int k = sd.Ss;
                    if (eobrun == 0) {
                        while (k <= sd.Se && !b.bad) {
                            const uint32_t a = ac_code(&at[0], b.peek());
                            if (!a) { b.bad = true; break; }
                            uint32_t r = (a >> 4) & 15; const uint32_t sz = a & 15;
                            b.skip(a >> 8);
                            if (sz > 1) { b.bad = true; break; }
                            if (sz == 0 && r < 15) { eobrun = (1u << r) + b.take(r); break; }   // (counts this block)
                            if (sz) b.skip(1);                       // the sign
                            while (k <= sd.Se) {                     // over r zeros; a correction bit at every non-zero on the way
                                if ((h >> k) & 1) b.skip(1);
                                else { if (r == 0) break; r--; }
                                k++;
                            }
                            if (sz) { if (k > sd.Se) { b.bad = true; break; } h |= 1ull << k; }
                            k++;
                        }
                    }
                    if (eobrun) {                                    // the rest of the block: corrections only
                        const uint64_t rest = k <= 63 ? (h & band & ~((1ull << k) - 1)) : 0;
                        b.skip((uint32_t)__builtin_popcountll(rest));
                        eobrun--;
                    }
                }
            }
        }
        if (b.bad) { E.clear(); return kOk; }                         // no entries from here on: later scans build on this one
    }
    return kOk;
}

struct IndexedPlan {
    RecordPlan P;
    uint32_t interval = 0;
    std::vector<std::vector<EntryPoint>> ent;                    // [n * kMaxScansPerFile]
};

inline int plan_record_indexed(const void* const* files, const size_t* sizes, uint32_t n, uint32_t interval, IndexedPlan* Q) {
    int rc = plan_record(files, sizes, n, &Q->P);
    if (rc) return rc;
    Q->interval = interval;
    Q->ent.assign((size_t)n * kMaxScansPerFile, std::vector<EntryPoint>());
    std::atomic<uint32_t> next(0);
    auto work = [&]() {
        for (;;) {
            const uint32_t i = next.fetch_add(1);
            if (i >= n) break;
            (void)find_entry_points((const uint8_t*)files[i], &Q->P.ends[(size_t)i * kMaxScansPerFile], Q->P.nscans[i], interval,
                                    &Q->ent[(size_t)i * kMaxScansPerFile]);   // (a file the walk refuses simply has no entries)
        }
    };
    const uint32_t nthreads = std::max(1u, std::min({16u, std::thread::hardware_concurrency(), n}));
    std::vector<std::thread> pool;
    for (uint32_t t = 1; t < nthreads; t++) pool.emplace_back(work);
    work();
    for (auto& t : pool) t.join();
    uint64_t entry_bytes_total = 0;
    for (const auto& e : Q->ent) entry_bytes_total += e.size() * (uint64_t)((!e.empty() && e[0].zero) ? kEntryBytesShort : kEntryBytes);
    const uint64_t raw = hdr_ecount_pos(n, Q->P.G, Q->P.G, 0);
    Q->P.header_bytes = (raw + 63) / 64 * 64;
    uint64_t payload = 0;
    for (uint32_t i = 0; i < n; i++) payload += sizes[i];
    Q->P.total = Q->P.header_bytes + payload + entry_bytes_total;
    if (Q->P.total >= (1ull << 32)) return kEUnsupported;
    return kOk;
}

inline void write_record_indexed(const IndexedPlan& Q, const void* const* files, const int32_t* labels, uint8_t* out) {
    const RecordPlan& P = Q.P;
    const uint32_t n = P.n, G = P.G;
    memset(out, 0, P.header_bytes);
    memcpy(out, "PCR1", 4);
    st_le32(out + 4, 2); st_le32(out + 8, n); st_le32(out + 12, G); st_le64(out + 16, P.header_bytes);
    st_le32(out + hdr_entry_interval_pos(n, G), Q.interval);
    uint64_t pos = P.header_bytes;
    for (uint32_t g = 0; g < G; g++) {
        for (uint32_t i = 0; i < n; i++) {
            uint32_t len = 0;
            if (g < P.nscans[i]) {
                const uint64_t* e = &P.ends[(size_t)i * kMaxScansPerFile];
                const uint64_t from = g ? e[g - 1] : 0;
                len = (uint32_t)(e[g] - from);
                memcpy(out + pos, (const uint8_t*)files[i] + from, len);
                pos += len;
            }
            st_le32(out + hdr_len_pos(n, G, g, i), len);
        }
        for (uint32_t i = 0; i < n; i++) {                          // the group's entries behind its regions
            const std::vector<EntryPoint>& E = Q.ent[(size_t)i * kMaxScansPerFile + g];
            uint8_t* c = out + hdr_ecount_pos(n, G, g, i);
            const bool brief = !E.empty() && E[0].zero;            // an AC scan: no DC predictions to carry
            const uint32_t field = (uint32_t)E.size() | (brief ? kEntryShortFlag : 0u);
            c[0] = (uint8_t)field; c[1] = (uint8_t)(field >> 8);
            for (const EntryPoint& e : E) {
                st_le32(out + pos, e.mcu); st_le32(out + pos + 4, e.bit);
                if (brief) { pos += kEntryBytesShort; continue; }
                for (int j = 0; j < 3; j++) { out[pos + 8 + 2 * j] = (uint8_t)(uint16_t)e.pred[j]; out[pos + 9 + 2 * j] = (uint8_t)((uint16_t)e.pred[j] >> 8); }
                out[pos + 14] = out[pos + 15] = 0;
                pos += kEntryBytes;
            }
        }
        st_le64(out + hdr_group_end_pos(g), pos);
    }
    for (uint32_t i = 0; i < n; i++) {
        st_le32(out + hdr_label_pos(G, i), labels ? (uint32_t)labels[i] : 0u);
        st_le32(out + hdr_nscans_pos(n, G, i), P.nscans[i]);
    }
}

// ---- progressive encoder --------------------------------------------------------------------------------
// A scan is first turned into tokens (Huffman symbol of one of two table slots + appended bits, or appended
// bits alone), the symbol counts give the scan its own optimal tables, then the tokens are written out.
struct Token { uint8_t slot; uint8_t sym; uint8_t nbits; uint16_t bits; };   // slot 0/1: Huffman table of the scan; 2: bits only; 3: restart marker number sym
constexpr uint8_t kRawBits = 2, kRestartMark = 3;

struct HuffSpec { uint8_t counts[17]; uint8_t symbols[256]; int nsym; uint16_t code[256]; uint8_t size[256]; };

// Code lengths from symbol counts, no code longer than 16 bits and none made of 1-bits only (the procedure of
// the JPEG specification's Annex K.2: a reserved extra symbol takes the all-ones code).
inline void build_table(const uint32_t freq_in[256], HuffSpec* H) {
    long freq[257]; int codesize[257], others[257];
    for (int i = 0; i < 256; i++) freq[i] = (long)freq_in[i];
    freq[256] = 1;
    for (int i = 0; i < 257; i++) { codesize[i] = 0; others[i] = -1; }
    for (;;) {
        int c1 = -1, c2 = -1;
        for (int i = 0; i < 257; i++) if (freq[i] > 0 && (c1 < 0 || freq[i] <= freq[c1])) c1 = i;      // least, ties: the larger index
        for (int i = 0; i < 257; i++) if (freq[i] > 0 && i != c1 && (c2 < 0 || freq[i] <= freq[c2])) c2 = i;
        if (c2 < 0) break;
        freq[c1] += freq[c2]; freq[c2] = 0;
        for (int v = c1;; v = others[v]) { codesize[v]++; if (others[v] < 0) { others[v] = c2; break; } }
        for (int v = c2; v >= 0; v = others[v]) codesize[v]++;
    }
    int bits[64] = {0};
    for (int i = 0; i < 257; i++) if (codesize[i]) bits[codesize[i] > 63 ? 63 : codesize[i]]++;
    for (int i = 63; i > 16; i--) {
        while (bits[i] > 0) {
            int j = i - 2;
            while (bits[j] == 0) j--;
            bits[i] -= 2; bits[i - 1] += 1; bits[j + 1] += 2; bits[j] -= 1;
        }
    }
    int longest = 16;
    while (longest > 0 && bits[longest] == 0) longest--;
    if (longest > 0) bits[longest]--;                          // the reserved symbol
    H->counts[0] = 0;
    for (int l = 1; l <= 16; l++) H->counts[l] = (uint8_t)bits[l];
    // symbols in order of code length; inside one length in order of value
    H->nsym = 0;
    for (int l = 1; l <= 63; l++)
        for (int s = 0; s < 256; s++) if (codesize[s] == l) H->symbols[H->nsym++] = (uint8_t)s;
    // canonical codes
    for (int s = 0; s < 256; s++) { H->code[s] = 0; H->size[s] = 0; }
    uint32_t code = 0; int k = 0;
    for (int l = 1; l <= 16; l++) {
        for (int c = 0; c < H->counts[l]; c++, k++) { H->code[H->symbols[k]] = (uint16_t)code; H->size[H->symbols[k]] = (uint8_t)l; code++; }
        code <<= 1;
    }
}

class BitWriter {
public:
    explicit BitWriter(std::vector<uint8_t>* out) : out_(out) {}
    void put(uint32_t bits, int n) {
        if (n == 0) return;
        acc_ = (acc_ << n) | (bits & ((1u << n) - 1u)); have_ += n;
        while (have_ >= 8) {
            const uint8_t b = (uint8_t)(acc_ >> (have_ - 8));
            out_->push_back(b);
            if (b == 0xFF) out_->push_back(0x00);
            have_ -= 8;
        }
    }
    void finish() { if (have_) put((1u << (8 - have_)) - 1u, 8 - have_); }      // pad with 1-bits
    void marker(uint8_t m) { finish(); out_->push_back(0xFF); out_->push_back(m); }
private:
    std::vector<uint8_t>* out_;
    uint64_t acc_ = 0; int have_ = 0;
};

struct Frame {
    int W, H, nc, hmax, vmax;
    int hs[kMaxComp], vs[kMaxComp], tq[kMaxComp], cid[kMaxComp];
    int bw[kMaxComp], bh[kMaxComp], cw[kMaxComp], ch[kMaxComp], mcux, mcuy;
    const int16_t* plane[kMaxComp];                            // [bh][bw][64], natural order inside a block
};

struct ScanSpec { int ns, comp[kMaxComp], Ss, Se, Ah, Al; };

inline int bit_length(int v) { int n = 0; while (v) { n++; v >>= 1; } return n; }

class ScanCoder {
public:
    // restart_mcus: MCUs of this scan per restart interval (0: no restart markers)
    ScanCoder(const Frame& F, const ScanSpec& S, uint32_t restart_mcus) : F_(F), S_(S), ri_(restart_mcus) {}
    std::vector<Token> tokens;

    void run() {
        size_t blocks = 0;
        for (int j = 0; j < S_.ns; j++) blocks += (size_t)F_.bw[S_.comp[j]] * F_.bh[S_.comp[j]];
        tokens.reserve(blocks * (S_.Ss == 0 ? 1 : 12));
        if (S_.Ss == 0) dc_scan(); else ac_scan();
    }

private:
    const Frame& F_; const ScanSpec& S_;
    uint32_t ri_, mcu_ = 0, marks_ = 0;                        // restart interval, MCUs begun, markers written
    int pred_[kMaxComp] = {0, 0, 0};                           // DC predictions
    // end-of-band run shared by the blocks of an AC scan, and the correction bits that wait behind it
    uint32_t eobrun_ = 0;
    std::vector<uint8_t> pending_;
    std::vector<uint8_t> corr_;                                // correction bits met since the last symbol of the current block

    void push(uint8_t slot, uint8_t sym, int nbits, uint32_t bits) { tokens.push_back(Token{slot, sym, (uint8_t)nbits, (uint16_t)(bits & 0xFFFFu)}); }
    void push_bits(const std::vector<uint8_t>& b) {
        size_t i = 0;
        while (i < b.size()) {
            uint32_t v = 0; int n = 0;
            while (n < 16 && i < b.size()) { v = (v << 1) | b[i++]; n++; }
            push(kRawBits, 0, n, v);
        }
    }
    const int16_t* block(int c, int row, int col) const { return F_.plane[c] + ((size_t)row * F_.bw[c] + col) * 64; }

    // A restart interval ends: whatever is pending goes out, a marker follows, predictions start again.
    void begin_mcu() {
        if (ri_ && mcu_ && mcu_ % ri_ == 0) {
            flush_eobrun();
            push(kRestartMark, (uint8_t)(marks_++ & 7), 0, 0);
            pred_[0] = pred_[1] = pred_[2] = 0;
        }
        mcu_++;
    }
    template <class Fn> void for_each_block(Fn fn) {
        if (S_.ns > 1) {
            for (int my = 0; my < F_.mcuy; my++) for (int mx = 0; mx < F_.mcux; mx++) {
                begin_mcu();
                for (int j = 0; j < S_.ns; j++) {
                    const int c = S_.comp[j];
                    for (int by = 0; by < F_.vs[c]; by++) for (int bx = 0; bx < F_.hs[c]; bx++)
                        fn(j, c, block(c, my * F_.vs[c] + by, mx * F_.hs[c] + bx));
                }
            }
        } else {
            const int c = S_.comp[0];
            for (int row = 0; row < F_.ch[c]; row++) for (int col = 0; col < F_.cw[c]; col++) { begin_mcu(); fn(0, c, block(c, row, col)); }
        }
    }

    void dc_scan() {
        for_each_block([&](int j, int c, const int16_t* b) {
            const int v = (int)b[0] >> S_.Al;                  // arithmetic shift: the point transform of DC
            if (S_.Ah == 0) {
                int diff = v - pred_[c]; pred_[c] = v;
                const int nb = bit_length(diff < 0 ? -diff : diff);
                push((uint8_t)(j == 0 ? 0 : 1), (uint8_t)nb, nb, (uint32_t)(diff < 0 ? diff - 1 : diff));
            } else {
                push(kRawBits, 0, 1, (uint32_t)(v & 1));
            }
        });
    }

    void flush_eobrun() {
        if (eobrun_ > 0) {
            const int n = bit_length((int)eobrun_) - 1;
            push(0, (uint8_t)(n << 4), n, eobrun_ - (1u << n));
            eobrun_ = 0;
        }
        if (!pending_.empty()) { push_bits(pending_); pending_.clear(); }
    }

    void ac_scan() {
        ZigzagTable zz;
        for_each_block([&](int, int, const int16_t* b) {
            if (S_.Ah == 0) ac_first_block(b, zz); else ac_refine_block(b, zz);
        });
        flush_eobrun();
    }

    void ac_first_block(const int16_t* b, const ZigzagTable& zz) {
        int run = 0;
        for (int k = S_.Ss; k <= S_.Se; k++) {
            const int c = b[zz.natural[k]];
            const int mag = (c < 0 ? -c : c) >> S_.Al;         // magnitudes are shifted, not the signed value
            if (mag == 0) { run++; continue; }
            flush_eobrun();
            while (run > 15) { push(0, 0xF0, 0, 0); run -= 16; }
            const int nb = bit_length(mag);
            push(0, (uint8_t)((run << 4) | nb), nb, (uint32_t)(c < 0 ? ~mag : mag));
            run = 0;
        }
        if (run > 0) { if (++eobrun_ == 0x7FFF) flush_eobrun(); }
    }

    void ac_refine_block(const int16_t* b, const ZigzagTable& zz) {
        int mag[64];
        int last_new = -1;                                     // last position that becomes non-zero in this scan
        for (int k = S_.Ss; k <= S_.Se; k++) {
            const int c = b[zz.natural[k]];
            mag[k] = (c < 0 ? -c : c) >> S_.Al;
            if (mag[k] == 1) last_new = k;
        }
        int run = 0;
        std::vector<uint8_t>& corr = corr_;
        corr.clear();
        for (int k = S_.Ss; k <= S_.Se; k++) {
            if (mag[k] == 0) { run++; continue; }
            while (run > 15 && k <= last_new) {                // sixteen zeros, only where a new coefficient still follows
                flush_eobrun();
                push(0, 0xF0, 0, 0);
                run -= 16;
                push_bits(corr); corr.clear();
            }
            if (mag[k] > 1) { corr.push_back((uint8_t)(mag[k] & 1)); continue; }     // known already: one more bit of it
            flush_eobrun();
            push(0, (uint8_t)((run << 4) | 1), 1, b[zz.natural[k]] < 0 ? 0u : 1u);
            push_bits(corr); corr.clear();
            run = 0;
        }
        if (run > 0 || !corr.empty()) {
            eobrun_++;
            pending_.insert(pending_.end(), corr.begin(), corr.end());
            if (eobrun_ == 0x7FFF) flush_eobrun();
        }
    }
};

inline void put_be16(std::vector<uint8_t>* o, uint32_t v) { o->push_back((uint8_t)(v >> 8)); o->push_back((uint8_t)v); }

inline void write_dht(std::vector<uint8_t>* o, int cls, int id, const HuffSpec& H) {
    o->push_back(0xFF); o->push_back(0xC4);
    put_be16(o, (uint32_t)(2 + 1 + 16 + H.nsym));
    o->push_back((uint8_t)((cls << 4) | id));
    for (int l = 1; l <= 16; l++) o->push_back(H.counts[l]);
    for (int k = 0; k < H.nsym; k++) o->push_back(H.symbols[k]);
}

// The script of the files written here (pcr_hist.h: the device counts the symbols of the same scans).
inline std::vector<ScanSpec> default_script(int nc) {
    std::vector<ScanSpec> s;
    for (int i = 0; i < script_scans(nc); i++) {
        const ScriptScan t = script_scan(nc, i);
        s.push_back(ScanSpec{t.ns, {t.comp[0], t.comp[1], t.comp[2]}, t.Ss, t.Se, t.Ah, t.Al});
    }
    return s;
}

// src: a JPEG file (baseline or progressive) whose frame header and quantisation tables are kept; coef: its
// quantised coefficients, component planes one after the other, each [bh][bw][64] in natural order over the
// MCU-padded block grid.  Appends the progressive file to *out.
// restart_interval: MCUs of each scan between restart markers (0: none; a scan of one component counts its blocks).
// counts (optional): the symbol counts of the scans, [scan][table slot][symbol] (kHistPerImage entries, as k_symbol_hist
// writes them), used for the Huffman tables instead of counting the tokens here.  counts_out (optional): receives the
// counts of the tokens; with it and out == nullptr nothing is written.
inline int transcode_progressive(const uint8_t* src, size_t src_bytes, const int16_t* coef, size_t coef_count, uint32_t restart_interval,
                                 std::vector<uint8_t>* out, const uint32_t* counts = nullptr, uint32_t* counts_out = nullptr) {
    std::vector<uint8_t> scratch;
    if (!out) out = &scratch;
    if (counts_out) memset(counts_out, 0, sizeof(uint32_t) * kHistPerImage);
    if (src_bytes >= (1ull << 32)) return kEUnsupported;
    if (restart_interval > 65535) return kERange;
    ParseState st;
    for (int a = 0; a < 2; a++) for (int b = 0; b < 4; b++) st.dht[a][b] = 0;
    st.ri = 0; st.have_frame = 0;
    ImgDesc img; memset(&img, 0, sizeof img);
    ScanDesc first; memset(&first, 0, sizeof first);
    int rc = parse_region(src, 0, (uint32_t)src_bytes, 1, &st, &img, &first, 0);      // up to the first scan header
    if (rc != kOk) return rc;
    Frame F;
    F.W = img.W; F.H = img.H; F.nc = img.nc; F.hmax = img.hmax; F.vmax = img.vmax; F.mcux = img.mcux; F.mcuy = img.mcuy;
    size_t need = 0;
    for (int c = 0; c < img.nc; c++) {
        F.hs[c] = img.hs[c]; F.vs[c] = img.vs[c]; F.tq[c] = img.tq[c]; F.cid[c] = img.cid[c];
        F.bw[c] = img.bw[c]; F.bh[c] = img.bh[c]; F.cw[c] = img.cw[c]; F.ch[c] = img.ch[c];
        if (!img.qoff[img.tq[c]]) return kEFormat;
        F.plane[c] = coef + need;
        need += (size_t)img.bw[c] * img.bh[c] * 64;
    }
    if (need != coef_count) return kERange;
    std::vector<uint8_t>& o = *out;
    o.push_back(0xFF); o.push_back(0xD8);
    bool done[4] = {false, false, false, false};
    for (int c = 0; c < img.nc; c++) {
        const int t = img.tq[c];
        if (done[t]) continue;
        done[t] = true;
        const int bytes = 64 * (img.qprec[t] + 1);
        o.push_back(0xFF); o.push_back(0xDB);
        put_be16(&o, (uint32_t)(2 + 1 + bytes));
        o.push_back((uint8_t)((img.qprec[t] << 4) | t));
        o.insert(o.end(), src + img.qoff[t], src + img.qoff[t] + bytes);
    }
    o.push_back(0xFF); o.push_back(0xC2);
    put_be16(&o, (uint32_t)(8 + 3 * img.nc));
    o.push_back(8); put_be16(&o, img.H); put_be16(&o, img.W); o.push_back((uint8_t)img.nc);
    for (int c = 0; c < img.nc; c++) { o.push_back((uint8_t)F.cid[c]); o.push_back((uint8_t)((img.nc == 1 ? 1 : F.hs[c]) << 4 | (img.nc == 1 ? 1 : F.vs[c]))); o.push_back((uint8_t)F.tq[c]); }
    if (restart_interval) {
        o.push_back(0xFF); o.push_back(0xDD);
        put_be16(&o, 4); put_be16(&o, restart_interval);
    }
    int scan_index = -1;
    for (const ScanSpec& S : default_script(img.nc)) {
        scan_index++;
        ScanCoder coder(F, S, restart_interval);
        coder.run();
        uint32_t freq[2][256];
        memset(freq, 0, sizeof freq);
        bool used[2] = {false, false};
        if (counts) {
            memcpy(freq, counts + (size_t)scan_index * kHistPerScan, sizeof freq);
            for (int s2 = 0; s2 < 2; s2++) for (int y = 0; y < 256; y++) if (freq[s2][y]) used[s2] = true;
            // (a token whose symbol the counts do not hold would get no code: refuse counts that do not fit the coefficients)
            for (const Token& t : coder.tokens) if (t.slot < kRawBits && freq[t.slot][t.sym] == 0) return kEFormat;
        } else {
            for (const Token& t : coder.tokens) if (t.slot < kRawBits) { freq[t.slot][t.sym]++; used[t.slot] = true; }
        }
        if (counts_out) memcpy(counts_out + (size_t)scan_index * kHistPerScan, freq, sizeof freq);
        HuffSpec H[2];
        const int cls = S.Ss == 0 ? 0 : 1;
        for (int s = 0; s < 2; s++) if (used[s]) { build_table(freq[s], &H[s]); write_dht(&o, cls, s, H[s]); }
        o.push_back(0xFF); o.push_back(0xDA);
        put_be16(&o, (uint32_t)(6 + 2 * S.ns));
        o.push_back((uint8_t)S.ns);
        for (int j = 0; j < S.ns; j++) {
            o.push_back((uint8_t)F.cid[S.comp[j]]);
            const int slot = (S.Ss == 0 && j > 0) ? 1 : 0;
            o.push_back((uint8_t)(cls == 0 ? (slot << 4) : slot));
        }
        o.push_back((uint8_t)S.Ss); o.push_back((uint8_t)S.Se); o.push_back((uint8_t)((S.Ah << 4) | S.Al));
        BitWriter bw(&o);
        for (const Token& t : coder.tokens) {
            if (t.slot == kRestartMark) { bw.marker((uint8_t)(0xD0 + t.sym)); continue; }
            if (t.slot < kRawBits) bw.put(H[t.slot].code[t.sym], H[t.slot].size[t.sym]);
            bw.put(t.bits, t.nbits);
        }
        bw.finish();
    }
    o.push_back(0xFF); o.push_back(0xD9);
    return kOk;
}

}  // namespace enc
}  // namespace pcr
