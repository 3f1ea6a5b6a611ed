// Entropy decoders with ONE LANE PER UNIT: the 64 lanes of a wavefront decode 64 different units (restart intervals or
// entry-point units) of the same kind of scan, each lane with its own bit buffer, Huffman table (the wavefront's copy, in
// LDS, of a table k_build_tables left in memory) and position in its image's coefficient plane.
//
// When they pay.  A wavefront that decodes one unit on the scalar ALU (pcr_entropy.h) spends about 14 scalar
// instructions per symbol, and the chip issues 256 of those per cycle: a throughput bound that a record with tens of
// thousands of units reaches.  A lane-per-unit wavefront is bound by latency instead: one symbol of every lane per trip
// round a dependent chain (buffer -> table entry -> lengths -> buffer) of one to two thousand cycles, but 64 symbols per
// trip, with a fifth of the instructions all told, and the trips of the wavefronts resident on a SIMD overlap.  With U units the scan takes about
// (symbols of the longest unit) x (chain latency), whatever U is, as long as the U / 64 wavefronts are resident at
// once; the host takes this path for launches with enough units (see lanes_pay in pcr_lib.hip) and the
// one-wavefront-per-unit kernels otherwise (few long units: plain records, small records).
//
// The price of 64 streams in one wavefront is that every branch some lane takes is paid by all: the symbol loop below
// is one straight line per symbol with selects, the rare cases (a code longer than 8 bits, a long end-of-band run that
// crosses rows) sit in short divergent regions.  The decoding procedure is the JPEG progressive mode's (the paper's
// Section 2: spectral selection and successive approximation); results are identical to the scalar decoders'.
#pragma once
#include "pcr_entropy.h"

namespace pcr {

// The decoders below are compiled for the host as well (one "lane", plain arrays for the rings): the CPU tests run them
// against the oracle and, on damaged input, under the sanitizers.
#if !defined(__HIPCC__)
struct uint4 { uint32_t x, y, z, w; };
struct uint2 { uint32_t x, y; };
#endif
// true if `v` holds in any lane of the wavefront that is still in the loop
PCR_HD bool any_lane(bool v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __any(v) != 0;
#else
    return v;
#endif
}
// Waits here for every load issued so far (device).  The wait the compiler would otherwise place at a loaded value's
// first use -- or at the first re-use of its register -- can land inside the symbol loop, and a wait for a load is a wait
// for every store issued before it as well: the loop would stand still for the round trip of its own stores in every
// trip.  (s_waitcnt vmcnt(0); the other counters are left at their maxima.)
PCR_HD void loads_arrived() {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0x0F70);
#endif
}
// bits [n, n + 32) of hi:lo counted from hi's top bit, n in 1..31 (one instruction on the device)
PCR_HD uint32_t funnel(uint32_t hi, uint32_t lo, uint32_t n) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_alignbit(hi, lo, 32u - n);
#else
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> (32u - n));
#endif
}

// The part of an AcTab (pcr_entropy.h) a lane decoder reads: everything before the pre-packed look-up of the window
// readers.  A wavefront keeps one per scan its lanes decode in LDS, and LDS is what bounds the number of resident
// wavefronts.
struct LaneTab {
    uint16_t lut[256];
    uint16_t lut2[128];
    uint32_t limit[9];
    uint16_t valptr[8];
    uint32_t sh2;
    uint8_t huffval[256];
};
constexpr uint32_t kLaneTabWords = sizeof(LaneTab) / 4;
static_assert(sizeof(LaneTab) == 1080 && offsetof(AcTab, lutp) >= sizeof(LaneTab) && offsetof(AcTab, lut2) == offsetof(LaneTab, lut2) &&
              offsetof(AcTab, limit) == offsetof(LaneTab, limit) && offsetof(AcTab, valptr) == offsetof(LaneTab, valptr) &&
              offsetof(AcTab, sh2) == offsetof(LaneTab, sh2) && offsetof(AcTab, huffval) == offsetof(LaneTab, huffval), "a LaneTab is the head of an AcTab");

// What a lane needs to know about its unit (AC scans: one component).
struct LaneUnit {
    const uint32_t* words;        // the scan's unstuffed data as big-endian words
    uint32_t bit0, bit1;          // the unit's bits [bit0, bit1) of that data
    uint32_t mcu0, mcu1, mcu_w;   // blocks [mcu0, mcu1) of the scan, mcu_w per row
    uint32_t bw;                  // blocks per row of the (padded) plane
    uint32_t Ss, Se, Al;
    int16_t* plane; uint32_t plane_elems;
    const LaneTab* tab;
    bool ok;
};

// A lane's view of its stream.  The next unread bit is the top bit of `hi`; hi:lo hold `have` valid bits (always more
// than 32 after top_up(), so that hi is a full look-ahead window; a symbol takes 31 at most).  A symbol's bits leave
// through a funnel shift (one instruction where a 64-bit shift of the pair and the copies around it are three or four).
//
// Words come from a ring of kRingWords words per lane in LDS, not from memory: the counter a wavefront waits on for a
// load is shared by all its lanes and returns in order, so a loop in which some lane or other fetches a word in every
// trip waits for memory in every trip.  The ring is filled for all lanes at once (refill: 16-byte chunks, as many as
// each lane has room for) whenever some lane is about to run short (short_of), every few dozen symbols; between two
// refills the loop reads no memory at all.
constexpr uint32_t kRingWords = 16, kRingChunks = kRingWords / 4;
struct LaneRing { uint4 chunk[kRingChunks][64]; };           // chunk c of lane i: its words 4c .. 4c+3 (mod kRingWords)

struct LaneStream {
    const uint4* base16;          // 16-byte aligned address at or before the unit's first word; word indices count from here
    uint32_t* ring;               // this lane's slot of chunk 0, as words (LDS); chunk c lies 256 c words further on
    uint32_t wi, wr;              // next word to enter the buffer; the ring holds the words before wr (a multiple of 4)
    uint32_t hi, lo; int have;
    int remain;                   // bits of the unit not consumed yet (negative: the decoder ran past the end)
    PCR_HD uint32_t ring_word(uint32_t w) const { return ring[((w >> 2) & (kRingChunks - 1)) * 256u + (w & 3u)]; }
    // Call with every lane that is still decoding.
    PCR_HD void refill() {
        const uint32_t room = (kRingWords - (wr - wi)) >> 2;  // whole chunks that fit
        const uint4* src = base16 + (wr >> 2);
        static_assert(kRingChunks == 4, "the chunks are spelled out (an array indexed in a loop ends up in scratch memory)");
        const uint4 v0 = src[0], v1 = src[1], v2 = src[2], v3 = src[3];   // (all four: the data stays readable well past a unit's end)
        loads_arrived();
        const uint32_t c0 = wr >> 2;
        if (room > 0) *reinterpret_cast<uint4*>(ring + ((c0 + 0) & 3u) * 256u) = v0;
        if (room > 1) *reinterpret_cast<uint4*>(ring + ((c0 + 1) & 3u) * 256u) = v1;
        if (room > 2) *reinterpret_cast<uint4*>(ring + ((c0 + 2) & 3u) * 256u) = v2;
        if (room > 3) *reinterpret_cast<uint4*>(ring + ((c0 + 3) & 3u) * 256u) = v3;
        wr += room * 4;
    }
    PCR_HD bool short_of(uint32_t words) const { return wr - wi < words; }
    PCR_HD void init(const uint32_t* words, uint32_t bit0, uint32_t bit1, LaneRing* rings, uint32_t lane) {
        const uint32_t* first = words + (bit0 >> 5);
        const uint32_t before = (uint32_t)(reinterpret_cast<uintptr_t>(first) & 15u) >> 2;   // words between the 16-byte boundary and the unit's first
        base16 = reinterpret_cast<const uint4*>(first - before);     // (pointer arithmetic: the address stays a global one)
        ring = reinterpret_cast<uint32_t*>(&rings->chunk[0][lane]);
        wi = before; wr = 0;
        refill();                                             // (wi < 4: all four chunks)
        const uint32_t off = bit0 & 31;
        const uint64_t buf = ((((uint64_t)ring_word(wi)) << 32) | ring_word(wi + 1)) << off;
        hi = (uint32_t)(buf >> 32); lo = (uint32_t)buf;
        have = 64 - (int)off; wi += 2;
        remain = (int)(bit1 - bit0);
    }
    PCR_HD void top_up() {
        if (have <= 32) {                                     // (then lo is empty)
            const uint64_t t = (uint64_t)ring_word(wi) << (32 - have);
            hi |= (uint32_t)(t >> 32); lo = (uint32_t)t;
            have += 32; wi++;
        }
    }
    PCR_HD uint32_t window() const { return hi; }
    PCR_HD void consume(uint32_t n) {                          // n in 1..31
        hi = funnel(hi, lo, n);
        lo <<= n; have -= (int)n; remain -= (int)n;
    }
    PCR_HD void consume_any(uint32_t n) {                      // n in 0..31
        hi = n ? funnel(hi, lo, n) : hi;
        lo <<= n; have -= (int)n; remain -= (int)n;
    }
};

// A code of more than 8 bits.  Some lane of 64 meets one in most trips, so the common case is kept short: the second
// look-up (pcr_entropy.h: indexed by the distance from the first long code, scaled to 128 entries) resolves every long
// code that owns a whole entry; the few that do not go through the canonical limits -- limit[L - 8] is the first
// left-aligned 16-bit value that is not a code of length <= L, so the length is 9 + the number of limits at or below
// the code.  Returns (length << 8) | symbol, or 0 if it is no code.
PCR_HD uint32_t lane_long_code(const LaneTab* t, uint32_t win) {
    const uint32_t c16 = win >> 16, lim8 = t->limit[0];
    const uint32_t i2 = (c16 - lim8) >> t->sh2;
    const bool longer = c16 >= lim8;
    uint32_t e = (longer && i2 < 128u) ? t->lut2[i2 & 127u] : 0u;
    if (longer && e == 0) {
        uint32_t L = 9, below = lim8;
#pragma unroll
        for (int q = 1; q <= 7; q++) {
            const uint32_t lim = t->limit[q];
            const bool over = c16 >= lim;
            L += over ? 1u : 0u; below = over ? lim : below;
        }
        const uint32_t idx = t->valptr[L - 9] + ((c16 - below) >> (16 - L));
        const uint32_t sym = t->huffval[idx & 255u];
        e = (c16 < t->limit[8] && idx < 256u) ? (L << 8) | sym : 0u;
    }
    return e;
}

// AC first scan (one component, band Ss..Se, point transform Al) of one unit.  Every coefficient the unit's symbols
// carry is stored (2 bytes); everything else in the plane was zero-filled before.  One symbol per trip, the three kinds
// of symbol (coefficient after a run, sixteen zeros, end of band) told apart by selects.
PCR_HD int lane_decode_ac_first(const LaneUnit& U, LaneRing* rings, uint32_t lane) {
    LaneStream st;
    st.init(U.words, U.bit0, U.bit1, rings, lane);
    const uint32_t Ss = U.Ss, Se = U.Se, mcu_w = U.mcu_w;
    uint32_t left = U.mcu1 - U.mcu0;                          // blocks of the unit not finished yet (the current one included)
    const uint32_t row0 = U.mcu0 / mcu_w;
    uint32_t col = U.mcu0 - row0 * mcu_w;
    uint32_t base = (row0 * U.bw + col) * 64;                 // element index of the current block
    const uint32_t row_skip = (U.bw - mcu_w) * 64;           // elements of the padded grid between two rows of the scan
    const float rcp_w = 1.0f / (float)mcu_w;
    uint32_t k = Ss, bad = 0;
    while (left != 0) {
        if (any_lane(st.short_of(2))) st.refill();              // (a trip takes one word at most)
        st.top_up();
        const uint32_t win = st.window();
        uint32_t e = U.tab->lut[win >> 24];
        if (e == 0) e = lane_long_code(U.tab, win);           // a code longer than 8 bits, or none
        bad |= e == 0 ? 1u : 0u;
        e = e ? e : (1u << 8);                                // (no code: one bit, nothing else; the lane stops below)
        const uint32_t len = e >> 8, r = (e >> 4) & 15u, s = e & 15u;
        const bool coef = s != 0, eob = s == 0 && r != 15u;
        const uint32_t nx = coef ? s : (eob ? r : 0u);        // appended bits: the value, or the length of an end-of-band run
        const uint32_t extra = ((win << len) >> 1) >> (31u - nx);
        st.consume(len + nx);
        k += eob ? 0u : (coef ? r : 16u);                     // the position the symbol lands on (sixteen zeros: passes)
        const uint32_t elem = base + k;
        const bool inside = k <= Se;
        if (coef && inside && elem < U.plane_elems) U.plane[elem] = (int16_t)((int16_t)extend(extra, (int)s) * (1 << U.Al));
        bad |= (coef && !inside) ? 1u : 0u;                   // a coefficient beyond the band
        bad |= st.remain < 0 ? 1u : 0u;                       // never walk beyond the unit's data
        k += coef ? 1u : 0u;
        const bool done = eob || k > Se;
        uint32_t adv = eob ? (1u << r) + extra : 1u;          // blocks to move on by: this one and the rest of an end-of-band run
        adv = adv < left ? adv : left;
        adv = done ? adv : 0u;
        left = bad ? 0u : left - adv;                         // stop at the first damaged block
        col += adv; base += adv * 64; k = done ? Ss : k;
        const bool wrap = col >= mcu_w;
        col -= wrap ? mcu_w : 0u; base += wrap ? row_skip : 0u;
        if (col >= mcu_w) {                                   // an end-of-band run over more than one row of blocks
            uint32_t q = (uint32_t)((float)col * rcp_w);      // rows passed, estimated: off by less than 1 + col / 2^22
            const uint32_t margin = 1u + (col >> 22);
            q = q > margin ? q - margin : 0;                  // never too high; the loop adds what is missing
            col -= q * mcu_w; base += q * row_skip;
            while (col >= mcu_w) { col -= mcu_w; base += row_skip; }
        }
    }
    return bad ? kEFormat : kOk;
}

// ---------------------------------------------------------------------------------------
// DC first scan of one unit (interleaved: up to three components, their blocks MCU by MCU; or one component, block by
// block over the blocks that cover its samples).  A unit's lanes belong to different images, each with its own two or
// three small tables, so the tables do not go through the job mechanism of the AC kernels: every lane makes its own,
// in LDS, in a form that needs no look-up memory worth the name -- the first sixteen codes of the table (more are no
// DC categories; the wavefront decoders drop them the same way) in code order, each as its left-aligned 16-bit value.
// Canonical codes in that form are increasing, so the code at the head of a 16-bit window w is the last one that is
// <= w: the lane counts them.  One symbol -- one block -- per trip.
// ---------------------------------------------------------------------------------------
constexpr uint32_t kLaneDcCodes = 16;
struct LaneDcTab {                                            // 80 bytes: read as 16-byte vectors, and five of them apart keeps 8 lanes on 32 banks
    uint16_t lim[kLaneDcCodes];                               // left-aligned code of entry i; 0xFFFF where there is none (no code is all ones)
    uint32_t len[2], cat[2];                                  // 4 bits per entry: code length - 1, category (entry i: bits 4 (i & 7) of word i >> 3)
    uint32_t n;                                               // entries
    uint32_t end;                                             // first left-aligned value that is no code of the (truncated) table
    uint32_t pad[6];
};
static_assert(sizeof(LaneDcTab) == 80, "LaneDcTab layout");
struct LaneDcTabs { LaneDcTab t[kMaxComp][64]; };            // [scan component][lane]

struct LaneDcUnit {
    const uint32_t* words; uint32_t bit0, bit1;               // as LaneUnit
    uint32_t mcu0, mcu1, mcu_w;
    uint32_t ns;                                              // components of the scan
    // per scan component 0, 1, 2 (single members, no arrays: a member picked by a run-time component number must be a
    // select between registers, and from an array the compiler makes it a load from a selected address in scratch memory):
    uint32_t hs0, hs1, hs2, vs0, vs1, vs2;                    // blocks per MCU (1 x 1 if ns == 1)
    uint32_t bw0, bw1, bw2;                                   // blocks per row of the component's plane
    uint32_t pblk0, pblk1, pblk2;                             // first block of its plane in the image's coefficient buffer
    int pred0, pred1, pred2;                                  // DC predictions at the unit's first MCU
    uint32_t Al;
    int16_t* dense;                                           // the image's compact copy of the DC coefficients: one value per block of the buffer
    int16_t* planes;                                          // the image's coefficient buffer (element 0 of every block), or null
    uint32_t nblocks;                                         // blocks of that buffer
    const uint8_t *def0, *def1, *def2;                        // each scan component's table definition: 16 counts, then the symbols in code order
    bool ok;
};

// The table of a definition (call per lane; t is the lane's own).
PCR_HD __attribute__((always_inline)) void lane_dctab_build(LaneDcTab* t, const uint8_t* bits_vals) {
    for (uint32_t i = 0; i < kLaneDcCodes; i++) t->lim[i] = 0xFFFFu;
    uint32_t code = 0, k = 0, n = 0, end = 0, len0 = 0, len1 = 0, cat0 = 0, cat1 = 0;
    for (uint32_t L = 1; L <= 16; L++) {
        const uint32_t cnt = bits_vals[L - 1];
        for (uint32_t j = 0; j < cnt; j++) {
            const uint32_t left = code << (16 - L);
            if (k < kLaneDcCodes && left < 0xFFFFu) {
                t->lim[k] = (uint16_t)left;
                const uint32_t sh = 4u * (k & 7u), c = bits_vals[16 + k] & 15u;
                if (k < 8) { len0 |= (L - 1u) << sh; cat0 |= c << sh; } else { len1 |= (L - 1u) << sh; cat1 |= c << sh; }
                end = left + (1u << (16 - L));
                n = k + 1;
            }
            code++; k++;
        }
        code <<= 1;
    }
    t->len[0] = len0; t->len[1] = len1; t->cat[0] = cat0; t->cat[1] = cat1; t->n = n;
    t->end = end > 0x10000u ? 0x10000u : end;
}

// v, as a value in a vector register whose origin the compiler does not look behind (see lane_decode_dc_first)
PCR_HD uint32_t lane_value(uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(v));
#endif
    return v;
}

PCR_HD __attribute__((always_inline)) int lane_decode_dc_first(const LaneDcUnit& U, LaneRing* rings, LaneDcTabs* tabs, uint32_t lane) {
    // The per-component members as plain values: picked by a run-time component number straight from U, the compiler
    // picks the member's address instead and loads from it, which puts the whole of U into scratch memory.
    const uint32_t hs0 = lane_value(U.hs0), hs1 = lane_value(U.hs1), hs2 = lane_value(U.hs2);
    const uint32_t vs0 = lane_value(U.vs0), vs1 = lane_value(U.vs1), vs2 = lane_value(U.vs2);
    const uint32_t bw0 = lane_value(U.bw0), bw1 = lane_value(U.bw1), bw2 = lane_value(U.bw2);
    const uint32_t pb0 = lane_value(U.pblk0), pb1 = lane_value(U.pblk1), pb2 = lane_value(U.pblk2);
    LaneStream st;
    st.init(U.words, U.bit0, U.bit1, rings, lane);
    static_assert(kMaxComp == 3, "the components are spelled out (an array indexed in a loop ends up in scratch memory)");
    lane_dctab_build(&tabs->t[0][lane], U.def0);
    if (U.ns > 1) lane_dctab_build(&tabs->t[1][lane], U.def1);
    if (U.ns > 2) lane_dctab_build(&tabs->t[2][lane], U.def2);
    const uint32_t n0 = hs0 * vs0, n01 = n0 + (U.ns > 1 ? hs1 * vs1 : 0u);
    const uint32_t bpm = n01 + (U.ns > 2 ? hs2 * vs2 : 0u);
    uint32_t left = U.mcu1 - U.mcu0;                          // MCUs not finished yet
    uint32_t my = U.mcu0 / U.mcu_w, mx = U.mcu0 - my * U.mcu_w, j = 0;
    int pred0 = U.pred0, pred1 = U.pred1, pred2 = U.pred2;
    uint32_t bad = 0;
    while (left != 0) {
        if (any_lane(st.short_of(2))) st.refill();
        st.top_up();
        const uint32_t win = st.window(), w16 = win >> 16;
        // the block: component c of the scan, block (by, bx) of its part of the MCU (sampling factors are 1 or 2)
        const uint32_t c = (j >= n0 ? 1u : 0u) + (j >= n01 ? 1u : 0u);
        const uint32_t jj = j - (c == 0 ? 0u : (c == 1 ? n0 : n01));
        const uint32_t hs = c == 0 ? hs0 : (c == 1 ? hs1 : hs2), vs = c == 0 ? vs0 : (c == 1 ? vs1 : vs2);
        const uint32_t bw = c == 0 ? bw0 : (c == 1 ? bw1 : bw2), p0 = c == 0 ? pb0 : (c == 1 ? pb1 : pb2);
        const uint32_t bx = jj & (hs - 1u), by = jj >> (hs - 1u);
        const uint32_t blk = p0 + (my * vs + by) * bw + mx * hs + bx;
        // the code: the last of the table's that is not above the window
        const LaneDcTab* T = &tabs->t[c][lane];
        // (three 16-byte reads that do not wait for the window: limits, limits, lengths and categories; then no further
        // trip to LDS stands between the window and the symbol)
        const uint4 la = *reinterpret_cast<const uint4*>(&T->lim[0]), lb = *reinterpret_cast<const uint4*>(&T->lim[8]);
        const uint4 lc = *reinterpret_cast<const uint4*>(&T->len[0]);
        const uint2 ne = *reinterpret_cast<const uint2*>(&T->n);
        const uint32_t lw[8] = {la.x, la.y, la.z, la.w, lb.x, lb.y, lb.z, lb.w};
        uint32_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;              // (four sums: no chain of sixteen additions)
#pragma unroll
        for (int q = 0; q < 8; q += 2) {
            c0 += (lw[q] & 0xFFFFu) <= w16 ? 1u : 0u; c1 += (lw[q] >> 16) <= w16 ? 1u : 0u;
            c2 += (lw[q + 1] & 0xFFFFu) <= w16 ? 1u : 0u; c3 += (lw[q + 1] >> 16) <= w16 ? 1u : 0u;
        }
        const uint32_t cnt = (c0 + c1) + (c2 + c3);           // codes at or below the window: the last of them is the one
        const uint32_t idx = (cnt - 1u) & 15u, sh = 4u * (idx & 7u);
        const bool code_ok = cnt != 0 && cnt <= ne.x && w16 < ne.y;
        const uint32_t len = code_ok ? (((idx < 8 ? lc.x : lc.y) >> sh) & 15u) + 1u : 1u, s = code_ok ? ((idx < 8 ? lc.z : lc.w) >> sh) & 15u : 0u;
        const uint32_t extra = ((win << len) >> 1) >> (31u - s);
        const int diff = extend(extra, (int)s);
        st.consume(len + s);
        bad |= code_ok ? 0u : 1u;
        bad |= st.remain < 0 ? 1u : 0u;                       // never walk beyond the unit's data
        int pred = c == 0 ? pred0 : (c == 1 ? pred1 : pred2);
        pred += diff;
        pred0 = c == 0 ? pred : pred0; pred1 = c == 1 ? pred : pred1; pred2 = c == 2 ? pred : pred2;
        if (!bad && blk < U.nblocks) {
            const int16_t v = (int16_t)(pred * (1 << U.Al));
            U.dense[blk] = v;
            if (U.planes) U.planes[(size_t)blk * 64] = v;
        }
        // on to the next block, MCU, row of MCUs
        j++;
        const bool mcu_done = j == bpm;
        j = mcu_done ? 0u : j;
        mx += mcu_done ? 1u : 0u;
        const bool row_done = mx == U.mcu_w;
        mx = row_done ? 0u : mx; my += row_done ? 1u : 0u;
        left -= mcu_done ? 1u : 0u;
        if (bad) left = 0;                                    // stop at the first damaged block
    }
    return bad ? kEFormat : kOk;
}

// ---------------------------------------------------------------------------------------
// AC refinement scan of one unit, complete in one pass: where the new coefficients go, their signs, and the correction
// bits.  The history of a block (which positions of the band are non-zero already) is read from the kRefHist word of
// the block's record, which k_refine_history has written for every block of the scan beforehand; like the stream
// words it comes through a small ring in LDS that all lanes fill at once.  Per block the lane leaves
//   [kRefNz]    positions that become non-zero,   [kRefSign]  their signs (1 = positive),
//   [kRefPlus]  the block's correction bits IN READING ORDER (first bit read = bit 0): k_refine_deal moves them to the
//               history positions they belong to afterwards, one lane per block.
// One trip of the loop is one symbol with the correction bits that follow it, or one block inside an end-of-band run
// (correction bits only).
// ---------------------------------------------------------------------------------------
constexpr uint32_t kHistRing = 4;
struct LaneHistRing { uint64_t h[kHistRing][64]; };

PCR_HD int lane_decode_ac_refine(const LaneUnit& U, uint64_t* recs, uint32_t nblk, LaneRing* rings, LaneHistRing* hring, uint32_t lane) {
    LaneStream st;
    st.init(U.words, U.bit0, U.bit1, rings, lane);
    const uint32_t Ss = U.Ss, Se = U.Se, mcu_w = U.mcu_w, row_skip = U.bw - mcu_w;
    const uint64_t band = band_mask((int)Ss, (int)Se);
    const uint32_t total = U.mcu1 - U.mcu0;
    uint32_t left = total;                                    // blocks of the unit not finished yet (the current one included)
    const uint32_t row0 = U.mcu0 / mcu_w;
    uint32_t col = U.mcu0 - row0 * mcu_w, blk = row0 * U.bw + col;
    const uint64_t* hist = recs + (size_t)kRefHist * nblk;
    // the cursor of the history fetches runs ahead of the decoder's
    uint32_t fcol = col, fblk = blk, fetched = 0, used_up = 0;
    auto fetch_history = [&]() {                              // every lane: as many blocks' words as its ring has room for
        static_assert(kHistRing == 4, "the entries are spelled out (an array indexed in a loop ends up in scratch memory)");
        uint32_t room = kHistRing - (fetched - used_up);
        room = room < total - fetched ? room : total - fetched;
        uint32_t b0 = fblk, b1, b2, b3;
        auto step = [&](uint32_t b) { uint32_t n = b + 1; fcol++; if (fcol == mcu_w) { fcol = 0; n += row_skip; } return n; };
        const uint32_t c0 = fcol;
        b1 = step(b0); b2 = step(b1); b3 = step(b2); const uint32_t b4 = step(b3);
        // (blocks past the unit's last are not read: the index is held at the last one wanted)
        const uint32_t l1 = room > 1 ? b1 : b0, l2 = room > 2 ? b2 : l1, l3 = room > 3 ? b3 : l2;
        const uint64_t v0 = hist[room > 0 ? b0 : blk];
        const uint64_t v1 = hist[room > 0 ? l1 : blk], v2 = hist[room > 0 ? l2 : blk], v3 = hist[room > 0 ? l3 : blk];
        loads_arrived();
        if (room > 0) hring->h[(fetched + 0) & 3u][lane] = v0;
        if (room > 1) hring->h[(fetched + 1) & 3u][lane] = v1;
        if (room > 2) hring->h[(fetched + 2) & 3u][lane] = v2;
        if (room > 3) hring->h[(fetched + 3) & 3u][lane] = v3;
        // the cursor moves on by `room` blocks
        fblk = room == 0 ? b0 : (room == 1 ? b1 : (room == 2 ? b2 : (room == 3 ? b3 : b4)));
        uint32_t fc = c0 + room;
        while (fc >= mcu_w) fc -= mcu_w;
        fcol = fc;
        fetched += room;
    };
    fetch_history();
    uint64_t h = hring->h[0][lane] & band, z = band & ~h;
    used_up = 1;
    uint64_t newm = 0, sgn = 0, corr = 0;
    uint32_t ncorr = 0, k = Ss, eobrun = 0, bad = 0;
    while (left != 0) {
        if (any_lane(st.short_of(4) || (fetched == used_up && fetched < total))) { st.refill(); fetch_history(); }
        st.top_up();
        const uint32_t win = st.window();
        uint32_t pos = Se;                                    // inside an end-of-band run: every correction of the block, nothing else
        uint32_t used = 0;                                    // bits of the window the symbol takes
        bool endb = true;
        if (eobrun == 0) {
            uint32_t e = U.tab->lut[win >> 24];
            if (e == 0) e = lane_long_code(U.tab, win);
            bad |= e == 0 ? 1u : 0u;
            e = e ? e : (1u << 8);
            const uint32_t len = e >> 8, r = (e >> 4) & 15u, s = e & 15u;
            bad |= s > 1 ? 1u : 0u;                           // sizes above 1 do not exist in a refinement scan
            const bool coef = s != 0, eob = s == 0 && r != 15u;
            const uint32_t extra = ((win << len) >> 1) >> (31u - (eob ? r : 0u));   // the length bits of an end-of-band run
            const uint32_t sign = (win << len) >> 31;
            // a coefficient takes the (r + 1)-th zero from k on, sixteen zeros land on the sixteenth (and leave it zero)
            const int p = nth_set_bit(z & (~0ull << k), coef ? r + 1u : 16u, 64);
            bad |= (coef && p == 64) ? 1u : 0u;               // a new coefficient with no zero left to take
            pos = (eob || p == 64) ? Se : (uint32_t)p;
            const uint64_t bit = coef ? 1ull << pos : 0ull;
            newm |= bit; sgn |= sign ? bit : 0ull;
            eobrun = eob ? (1u << r) + extra : 0u;
            used = len + (coef ? 1u : (eob ? r : 0u));
            endb = eob;
        }
        // the correction bits of the history positions from k to pos follow: mostly a few, inside the window still
        uint32_t m = (uint32_t)__builtin_popcountll(h & (~0ull << k) & ((2ull << pos) - 1ull));
        if (used + m <= 31u) {
            corr |= (uint64_t)(bitrev32(win << used) & ((1u << m) - 1u)) << ncorr;
            ncorr += m;
            st.consume_any(used + m);
        } else {
            st.consume_any(used);
            while (m) {
                st.top_up();
                const uint32_t t = m < 31u ? m : 31u;
                corr |= (uint64_t)(bitrev32(st.window()) & ((1u << t) - 1u)) << ncorr;
                ncorr += t; m -= t;
                st.consume(t);
            }
        }
        k = pos + 1;
        bad |= st.remain < 0 ? 1u : 0u;
        if (endb || k > Se) {                                 // the block is complete
            uint64_t* rec = recs + blk;
            rec[(size_t)kRefNz * nblk] = newm; rec[(size_t)kRefSign * nblk] = sgn; rec[(size_t)kRefPlus * nblk] = corr;
            eobrun -= eobrun ? 1u : 0u;                       // (a run counts the block it starts in)
            left--;
            blk++; if (++col == mcu_w) { col = 0; blk += row_skip; }
            if (left != 0) { h = hring->h[used_up & 3u][lane] & band; used_up++; z = band & ~h; }
            newm = 0; sgn = 0; corr = 0; ncorr = 0; k = Ss;
        }
        if (bad) left = 0;                                    // stop at the first damaged block
    }
    return bad ? kEFormat : kOk;
}

}  // namespace pcr
