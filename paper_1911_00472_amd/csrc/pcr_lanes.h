// Entropy decoders with ONE LANE PER UNIT: the 64 lanes of a wavefront decode 64 different units (restart intervals or
// entry-point units) of the same kind of scan, each lane with its own bit buffer, Huffman table (read from the tables
// k_build_tables left in memory) and position in its image's coefficient plane.
//
// When they pay.  A wavefront that decodes one unit on the scalar ALU (pcr_entropy.h) spends about 14 scalar
// instructions per symbol, and the chip issues 256 of those per cycle: a throughput bound that a record with tens of
// thousands of units reaches.  A lane-per-unit wavefront is bound by latency instead: one symbol of every lane per trip
// round a dependent chain (buffer -> table entry -> lengths -> buffer) of some hundred cycles, but 64 symbols per trip,
// and the trips of the wavefronts resident on a SIMD overlap.  With U units the scan takes about
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

#if defined(__HIPCC__)

// What a lane needs to know about its unit (AC scans: one component).
struct LaneUnit {
    const uint32_t* words;        // the scan's unstuffed data as big-endian words
    uint32_t bit0, bit1;          // the unit's bits [bit0, bit1) of that data
    uint32_t mcu0, mcu1, mcu_w;   // blocks [mcu0, mcu1) of the scan, mcu_w per row
    uint32_t bw;                  // blocks per row of the (padded) plane
    uint32_t Ss, Se, Al;
    int16_t* plane; uint32_t plane_elems;
    const AcTab* tab;
    bool ok;
};

// A lane's view of its stream.  The next unread bit is the top bit of `hi`; hi:lo hold `have` valid bits (always more
// than 32 after top_up(), so that hi is a full look-ahead window; a symbol takes 31 at most).  A symbol's bits leave
// through a funnel shift (one instruction; 64-bit shifts run at a quarter of the rate).
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
    PCR_D uint32_t ring_word(uint32_t w) const { return ring[((w >> 2) & (kRingChunks - 1)) * 256u + (w & 3u)]; }
    // Call with every lane that is still decoding; `mine`: this lane takes part.
    PCR_D void refill() {
        const uint32_t room = (kRingWords - (wr - wi)) >> 2;  // whole chunks that fit
        const uint4* src = base16 + (wr >> 2);
        static_assert(kRingChunks == 4, "the chunks are spelled out (an array indexed in a loop ends up in scratch memory)");
        const uint4 v0 = src[0], v1 = src[1], v2 = src[2], v3 = src[3];   // (all four: the data stays readable well past a unit's end)
        const uint32_t c0 = wr >> 2;
        if (room > 0) *reinterpret_cast<uint4*>(ring + ((c0 + 0) & 3u) * 256u) = v0;
        if (room > 1) *reinterpret_cast<uint4*>(ring + ((c0 + 1) & 3u) * 256u) = v1;
        if (room > 2) *reinterpret_cast<uint4*>(ring + ((c0 + 2) & 3u) * 256u) = v2;
        if (room > 3) *reinterpret_cast<uint4*>(ring + ((c0 + 3) & 3u) * 256u) = v3;
        wr += room * 4;
    }
    PCR_D bool short_of(uint32_t words) const { return wr - wi < words; }
    PCR_D void init(const uint32_t* words, uint32_t bit0, uint32_t bit1, LaneRing* rings, uint32_t lane) {
        const uint32_t* first = words + (bit0 >> 5);
        const uintptr_t a = reinterpret_cast<uintptr_t>(first);
        base16 = reinterpret_cast<const uint4*>(a & ~(uintptr_t)15);
        ring = reinterpret_cast<uint32_t*>(&rings->chunk[0][lane]);
        wi = (uint32_t)(a & 15) >> 2; wr = 0;
        refill();                                             // (wi < 4: all four chunks)
        const uint32_t off = bit0 & 31;
        const uint64_t buf = ((((uint64_t)ring_word(wi)) << 32) | ring_word(wi + 1)) << off;
        hi = (uint32_t)(buf >> 32); lo = (uint32_t)buf;
        have = 64 - (int)off; wi += 2;
        remain = (int)(bit1 - bit0);
    }
    PCR_D void top_up() {
        if (have <= 32) {                                     // (then lo is empty)
            const uint64_t t = (uint64_t)ring_word(wi) << (32 - have);
            hi |= (uint32_t)(t >> 32); lo = (uint32_t)t;
            have += 32; wi++;
        }
    }
    PCR_D uint32_t window() const { return hi; }
    PCR_D void consume(uint32_t n) {                          // n in 1..31
        hi = __builtin_amdgcn_alignbit(hi, lo, 32u - n);
        lo <<= n; have -= (int)n; remain -= (int)n;
    }
};

// A code of more than 8 bits, by the canonical limits (pcr_entropy.h: limit[L - 8] is the first left-aligned 16-bit
// value that is not a code of length <= L): its length is 9 + the number of limits at or below it; no branches, since
// some lane of 64 meets such a code in every other symbol.  Returns (length << 8) | symbol, or 0 if it is no code.
PCR_D uint32_t lane_long_code(const AcTab* t, uint32_t win) {
    const uint32_t c16 = win >> 16;
    uint32_t L = 9, below = t->limit[0];                      // below: the limit under the code's length
#pragma unroll
    for (int q = 1; q <= 7; q++) {
        const uint32_t lim = t->limit[q];
        const bool over = c16 >= lim;
        L += over ? 1u : 0u; below = over ? lim : below;
    }
    const uint32_t idx = t->valptr[L - 9] + ((c16 - below) >> (16 - L));
    const uint32_t sym = t->huffval[idx & 255u];
    return (c16 < t->limit[8] && idx < 256u) ? (L << 8) | sym : 0u;
}

// AC first scan (one component, band Ss..Se, point transform Al) of one unit.  Every coefficient the unit's symbols
// carry is stored (2 bytes); everything else in the plane was zero-filled before.  One symbol per trip, the three kinds
// of symbol (coefficient after a run, sixteen zeros, end of band) told apart by selects.
PCR_D int lane_decode_ac_first(const LaneUnit& U, LaneRing* rings, uint32_t lane) {
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
        if (__any(st.short_of(2))) st.refill();              // (a trip takes one word at most)
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

#endif  // __HIPCC__

}  // namespace pcr
