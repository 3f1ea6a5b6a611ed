// Corruption sweep under AddressSanitizer / UndefinedBehaviorSanitizer, CPU only.  Reads a record file and the JPEG
// files it was made of, damages copies of them in seeded ways (bit flips, byte runs, truncations, header fields), and
// pushes every damaged copy through the host-side code that parses untrusted bytes: the CPU oracle, the library's
// lane code as compiled for the CPU (marker parser, Huffman tables, scan decoders of both shapes: emul_decode_record), and the
// library's record writer with its entry-point walk and scan splitter.  Nothing is checked but "no sanitizer
// report": results of damaged input are allowed to be errors or garbage.  Test infrastructure only.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../paper_1911_00472_amd/csrc/pcr_encode.h"

extern "C" {
int emul_decode_record(const uint8_t* rec, size_t nbytes, int k, int64_t want_img, int16_t* coef_out, uint8_t* pix_out, int* W, int* H, int* C);
void emul_set_lane_decoders(int on);
int orc_record_header(const uint8_t* rec, size_t nbytes, uint32_t* n, uint32_t* G, uint64_t* header_bytes, int* k_avail);
typedef struct { int W, H, nc, hs[3], vs[3], bw[3], bh[3], nscans, progressive; } orc_info_t;
int orc_record_image_info(const uint8_t* rec, size_t nbytes, uint32_t i, orc_info_t* info);
int orc_decode_record_image(const uint8_t* rec, size_t nbytes, uint32_t i, int k, int upsample, int idct, int16_t* coef, uint8_t* pix);
int orc_reassemble(const uint8_t* rec, size_t nbytes, uint32_t i, int k, uint8_t* dst, size_t cap, size_t* out_len);
int orc_decode_smooth(const uint8_t* jpg, size_t n, int16_t* coef, uint8_t* pix);
}

static uint64_t rng_state = 1;
static uint32_t rnd() { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17; return (uint32_t)(rng_state >> 16); }

static std::vector<uint8_t> read_file(const char* path) {
    std::vector<uint8_t> v;
    FILE* f = fopen(path, "rb");
    if (!f) { fprintf(stderr, "cannot open %s\n", path); exit(2); }
    uint8_t buf[65536]; size_t n;
    while ((n = fread(buf, 1, sizeof buf, f)) > 0) v.insert(v.end(), buf, buf + n);
    fclose(f);
    return v;
}

static void damage(std::vector<uint8_t>& d, int kind, size_t protect_from, size_t protect_to) {
    if (d.empty()) return;
    auto pos = [&]() { size_t p = rnd() % d.size(); return p; };
    switch (kind) {
        case 0: for (int j = 0; j < 1 + (int)(rnd() % 4); j++) d[pos()] ^= (uint8_t)(1u << (rnd() % 8)); break;         // bit flips anywhere
        case 1: { size_t p = pos(); for (size_t j = p; j < d.size() && j < p + 1 + rnd() % 40; j++) d[j] = (uint8_t)rnd(); break; }   // a run of noise
        case 2: d.resize(1 + rnd() % d.size()); break;                                                                    // truncation
        case 3: { size_t span = protect_to > protect_from ? protect_to - protect_from : 1; d[(protect_from + rnd() % span) % d.size()] = (uint8_t)rnd(); break; }  // inside the headers
        case 4: { size_t p = pos(); d[p] = 0xFF; if (p + 1 < d.size()) d[p + 1] = (uint8_t)(0xC0 + rnd() % 0x40); break; }  // a stray marker
        default: { size_t p = pos(); size_t n = 1 + rnd() % 16; if (p + n < d.size()) d.erase(d.begin() + (long)p, d.begin() + (long)(p + n)); break; }   // bytes removed
    }
}

static void through_the_decoders(const std::vector<uint8_t>& rec) {
    uint32_t n = 0, G = 0; uint64_t hb = 0; int kav = 0;
    if (orc_record_header(rec.data(), rec.size(), &n, &G, &hb, &kav) != 0 || n == 0 || n > 64 || G > 64) return;   // (keep the sweep bounded)
    for (uint32_t i = 0; i < n; i++) {
        orc_info_t info;
        std::vector<int16_t> coef; std::vector<uint8_t> pix;
        const bool known = orc_record_image_info(rec.data(), rec.size(), i, &info) == 0 && info.W > 0 && info.W <= 4096 && info.H > 0 && info.H <= 4096;
        if (known) {
            size_t cc = 0;
            for (int c = 0; c < info.nc && c < 3; c++) cc += (size_t)info.bw[c] * info.bh[c] * 64;
            coef.resize(cc + 64); pix.resize((size_t)info.W * info.H * 3 + 64);
        }
        for (int k = 1; k <= kav; k += (kav > 4 ? 3 : 1)) {
            size_t len = 0;
            std::vector<uint8_t> tmp(rec.size() + 2);
            (void)orc_reassemble(rec.data(), rec.size(), i, k, tmp.data(), tmp.size(), &len);
            if (!known) continue;
            (void)orc_decode_record_image(rec.data(), rec.size(), i, k, 0, 0, coef.data(), pix.data());
            if (k <= 3) (void)orc_decode_smooth(tmp.data(), len, coef.data(), pix.data());      // (the first groups are where components hold only DC)
            int W = 0, H = 0, C = 0;
            for (int lanes = 0; lanes < 2; lanes++) {                    // both shapes of AC decoder (pcr_entropy.h, pcr_lanes.h)
                emul_set_lane_decoders(lanes);
                (void)emul_decode_record(rec.data(), rec.size(), k, (int64_t)i, coef.data(), pix.data(), &W, &H, &C);
            }
        }
    }
}

int main(int argc, char** argv) {
    if (argc < 4) { fprintf(stderr, "usage: sweep <seed> <rounds> <record> [jpeg files...]\n"); return 2; }
    rng_state = (uint64_t)strtoull(argv[1], nullptr, 10) * 0x9E3779B97F4A7C15ull + 1;
    const int rounds = atoi(argv[2]);
    const std::vector<uint8_t> record = read_file(argv[3]);
    std::vector<std::vector<uint8_t>> files;
    for (int a = 4; a < argc; a++) files.push_back(read_file(argv[a]));
    through_the_decoders(record);                                       // the undamaged input first
    uint64_t hb = record.size() >= 24 ? pcr::ld_le64(record.data() + 16) : 24;
    for (int r = 0; r < rounds; r++) {
        std::vector<uint8_t> bad = record;
        damage(bad, (int)(rnd() % 6), 0, (size_t)hb);
        through_the_decoders(bad);
        if (files.empty()) continue;
        // the record writer (scan splitter, entry-point walk) on damaged files
        std::vector<std::vector<uint8_t>> fb = files;
        std::vector<uint8_t>& victim = fb[rnd() % fb.size()];
        damage(victim, (int)(rnd() % 6), 0, 600);
        std::vector<const void*> ptrs; std::vector<size_t> sizes;
        for (auto& f : fb) { ptrs.push_back(f.data()); sizes.push_back(f.size()); }
        pcr::enc::IndexedPlan Q;
        if (pcr::enc::plan_record_indexed(ptrs.data(), sizes.data(), (uint32_t)fb.size(), 1 + rnd() % 200, &Q) == 0) {
            std::vector<uint8_t> out(Q.P.total);
            pcr::enc::write_record_indexed(Q, ptrs.data(), nullptr, out.data());
            if (r % 4 == 0) through_the_decoders(out);                   // what the writer made of a damaged file goes through the decoders as well
        }
    }
    printf("sweep ok: %d rounds\n", rounds);
    return 0;
}
