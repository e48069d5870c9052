// Pieces of the chunked Huffman encoder (COMET Sec. 4.1, last step of the pipeline) that the
// encode kernels and the single-pass compressor share: the encode table view, the prefix sum
// inside the lane group of a chunk, the test for chunks that take no words.
#pragma once
#include "comet_kernels.h"

namespace comet {

namespace {

// The encode table as the encoders see it.  TM 1 (or true): the whole table is in LDS.  Keeping global loads out
// of that variant matters: a load inside the loop would make every iteration wait for the stores of the previous
// one.  TM 0 (or false): the entries [lo, lo + n) are in LDS, the others are looked up in global memory.  TM 2: as
// TM 0, but every symbol that has a code word lies in [lo, lo + n), but for the escape symbol 0, whose entry is kept
// behind the cached ones (k_codebook says whether that holds: Control::enc_in_window); again no global loads.
template <int TM>
struct TableView {
    const uint64_t *lds;
    const uint64_t *glob;
    uint32_t lo, n, nbins;
    // A code outside the alphabet cannot come from the quantise kernel; it reads the entry that follows the
    // cached part: zero (length 0: the symbol contributes no bits), in TM 2 the escape symbol's.
    __device__ inline uint32_t index(uint32_t code) const {
        if (TM == 1) return code < nbins ? code : nbins;
        const uint32_t i = code - lo;                 // (TM 2; a code below lo wraps to a large number)
        return i < n ? i : n;
    }
    __device__ inline uint64_t full(uint32_t code) const {
        if (TM != 0) return lds[index(code)];
        if (code >= nbins) return 0ull;
        const uint32_t i = code - lo;
        return (i < n) ? lds[i] : glob[code];
    }
    // length only
    __device__ inline uint32_t length(uint32_t code) const {
        if (TM != 0) return reinterpret_cast<const uint32_t *>(lds)[2u * index(code)] & 63u;
        return (uint32_t)full(code) & 63u;
    }
};

// The code lengths alone, one byte each, of the symbols [lo, lo + n) in LDS; behind them the escape symbol's.  For the
// count kernel when every symbol that occurs lies in that range (Control::len_in_window): eight times the symbols of the
// encode table's cached part in the same LDS, and no look-up in global memory.
struct LengthView {
    const uint8_t *lds;
    uint32_t lo, n;
    __device__ inline uint32_t length(uint32_t code) const {
        const uint32_t i = code - lo;                 // (a code below lo wraps to a large number)
        return lds[i < n ? i : n];
    }
};

// inclusive prefix sum inside groups of LPC = 16, 32 or 64 adjacent lanes (DPP, no LDS)
template <int LPC>
__device__ inline uint32_t group_incl_scan(uint32_t v) {
    int32_t x = (int32_t)v;
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, true);    // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, true);    // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, true);    // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, true);    // row_shr:8
    if (LPC >= 32) x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1, 3
    if (LPC >= 64) x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2, 3
    return (uint32_t)x;
}

// Container version 2 (sparse activations behind ReLU, COMET Sec. 4.2): which chunks of the step hold
// nothing but the centre code and therefore take no words; true for the lanes of such a chunk.  left:
// symbols of the step that exist (256 except at the end of the tensor; positions past the end do not count).
template <int LPC>
__device__ inline bool chunk_is_centre_only(uint2 v, uint32_t zero_pair, uint32_t lane, uint32_t left) {
    bool mine = v.x == zero_pair && v.y == zero_pair;
    if (left < 256u) {
        const uint32_t centre = zero_pair & 0xffffu;
        mine = true;
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
            const uint32_t w = (j < 2) ? v.x : v.y;
            const uint32_t c = (j & 1) ? (w >> 16) : (w & 0xffffu);
            mine = mine && (lane * 4u + j >= left || c == centre);
        }
    }
    const uint64_t all = wave_ballot(mine);
    constexpr uint64_t grp = LPC == 64 ? ~0ull : ((1ull << (LPC & 63)) - 1ull);
    return ((all >> ((lane / LPC) * LPC)) & grp) == grp;
}

__device__ inline uint32_t code_of(uint2 v, int j) {
    const uint32_t w = (j < 2) ? v.x : v.y;
    return (j & 1) ? (w >> 16) : (w & 0xffffu);
}


// ---------------------------------------------------------------------------------------------
// The encoder of the single-pass compressor (compression with a given code book): a wavefront
// that quantises a run of rows keeps its codes in a ring in LDS and encodes them 256 at a time,
// with the lane layout of k_encode_pack, as soon as they are there.  The words go to a work area
// of the run (positions relative to the run, like the chunk offsets it writes); a small kernel
// moves them to their place once the sizes of all runs and the record count are known.
// ---------------------------------------------------------------------------------------------
constexpr uint32_t kEncOob = 0x80000000u;       // byte offset beyond every buffer
struct RunEncoder {
    const uint16_t *ring;       // LDS: kEncRingSyms codes, element e of the run at e % kEncRingSyms
    uint32_t *buf;              // LDS: assembly buffer of one step, kEncRunBufWords words, zero between steps
    __amdgpu_buffer_rsrc_t r_words;   // global: the run's words (as many as fit)
    uint32_t cap_words;
    __amdgpu_buffer_rsrc_t r_chunk;   // global: the chunk table entries of the run's chunks
    uint32_t zero_pair;         // container version 2: (centre << 16) | centre, else 0
    uint32_t consumed = 0;      // symbols encoded so far (a multiple of 256 until the run's last step)
    uint32_t wrun = 0;          // words written so far
    bool overflow = false;

    // One step: the next `left` (<= 256) symbols of the ring.
    template <int S, bool FULLTBL>
    __device__ inline void step(const TableView<FULLTBL> &tbl, uint32_t lane, uint32_t left) {
        constexpr int LPC = S / 4;
        constexpr int CPS = 256 / S;
        const uint32_t rp = consumed & (kEncRingSyms - 1u);
        const uint2 v = *reinterpret_cast<const uint2 *>(ring + rp + lane * 4u);
        uint64_t cw[4];
        uint32_t len[4], bits = 0;
        uint64_t acc = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint64_t e = tbl.full(code_of(v, j));
            if (__builtin_expect(left < 256u, 0)) e = (lane * 4u + (uint32_t)j < left) ? e : 0ull;   // (uniform; the run's last step only)
            len[j] = (uint32_t)e & 63u;
            cw[j] = e >> 6;
            bits += len[j];
            acc = (acc << len[j]) | cw[j];
        }
        if (zero_pair && chunk_is_centre_only<LPC>(v, zero_pair, lane, left)) bits = 0;
        const uint32_t incl = group_incl_scan<LPC>(bits);
        const uint32_t g = lane / LPC;
        uint32_t wbase = 0, total_words = 0;
#pragma unroll
        for (int k = 0; k < CPS; ++k) {
            const uint32_t wk = ((uint32_t)__builtin_amdgcn_readlane((int)incl, k * LPC + LPC - 1) + 31u) >> 5;
            if ((uint32_t)k == g) wbase = total_words;
            total_words += wk;
        }
        // (buffer stores that every lane issues, with an offset out of range where there is nothing to store: a
        // store inside a branch would make the quantise loop around this wait for all its loads at every turn)
        __builtin_amdgcn_raw_buffer_store_b32(wrun + wbase, r_chunk,
                                              ((lane % LPC) == 0u && g * (uint32_t)S < left) ? (int)((consumed / (uint32_t)S + g) * 4u) : (int)kEncOob, 0, 0);
        uint32_t p = wbase * 32u + incl - bits;
        auto place = [&](uint64_t t, uint32_t L, uint32_t at) {
            const uint32_t sh = at & 31u, w = at >> 5;
            const uint64_t hi = t >> sh;
            atomicOr(&buf[w], (uint32_t)(hi >> 32));
            atomicOr(&buf[w + 1], (uint32_t)hi);
            if (L + sh > 64u) atomicOr(&buf[w + 2], (uint32_t)((t << (64u - sh)) >> 32));
        };
        if (bits <= 64u) {
            place(bits ? acc << (64u - bits) : 0ull, bits, p);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t L = len[j];
                if (L) place(cw[j] << (64u - L), L, p);
                p += L;
            }
        }
        wave_lds_fence();
        // the step's words leave: 128 of them (16 bits per symbol) with two stores of every lane, the rare rest in a loop;
        // what lies beyond the run's work area is dropped by the buffer's range check
#pragma unroll
        for (uint32_t k0 = 0; k0 < 2u * kWave; k0 += kWave) {
            const uint32_t k = k0 + lane;
            const uint32_t word = buf[k];
            buf[k] = 0;
            __builtin_amdgcn_raw_buffer_store_b32(word, r_words, k < total_words ? (int)((wrun + k) * 4u) : (int)kEncOob, 0, 0);
        }
        if (__builtin_expect(total_words > 2u * kWave, 0)) {
            for (uint32_t k = 2u * kWave + lane; k < total_words; k += kWave) {
                const uint32_t word = buf[k];
                buf[k] = 0;
                __builtin_amdgcn_raw_buffer_store_b32(word, r_words, (int)((wrun + k) * 4u), 0, 0);
            }
        }
        if (wrun + total_words > cap_words) overflow = true;
        wave_lds_fence();
        wrun += total_words;
        consumed += left;
    }

    // Everything that can be encoded of the `produced` symbols the ring has received: whole steps, and at
    // the end of the run (final) the rest.
    template <int S, bool FULLTBL>
    __device__ inline void drain(const TableView<FULLTBL> &tbl, uint32_t lane, uint32_t produced, bool final) {

        while (produced - consumed >= 256u) step<S, FULLTBL>(tbl, lane, 256u);
        if (final && consumed < produced) step<S, FULLTBL>(tbl, lane, produced - consumed);
    }
};

}  // namespace

}  // namespace comet
