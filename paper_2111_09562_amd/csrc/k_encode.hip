// Chunked Huffman encode (COMET Sec. 4.1, last step of the modified cuSZ
// pipeline).  One lane encodes one chunk of chunk_syms consecutive codes; a
// workgroup of 256 lanes takes tiles of 256 chunks by ticket.
//   stage : the tile's codes are copied global -> LDS with coalesced 16-byte
//           loads, every chunk padded by 8 codes so that the per-lane 16-byte
//           LDS reads that follow hit distinct banks;
//   pass A: each lane sums the code lengths of its chunk -> 32-bit words;
//   scan  : workgroup scan of the word counts + chained scan over tiles gives
//           every chunk its word offset in the payload (deterministic layout);
//   pass B: each lane packs its codes most-significant-bit first through a
//           64-bit buffer and writes whole 32-bit words; the last word of a chunk
//           is zero padded.
// The encode table ((code << 6) | length per symbol) is cached in LDS for the
// bins around the centre; other symbols are looked up in global memory.
#include "comet_kernels.h"

namespace comet {

namespace {

struct TableView {
    const uint64_t *lds;
    const uint64_t *glob;
    uint32_t lo, n;
    __device__ inline uint64_t full(uint32_t code) const {
        const uint32_t i = code - lo;
        return (i < n) ? lds[i] : glob[code];
    }
    __device__ inline uint32_t length(uint32_t code) const {
        const uint32_t i = code - lo;
        return (uint32_t)((i < n) ? reinterpret_cast<const uint32_t *>(lds)[2 * i] : (uint32_t)glob[code]) & 63u;
    }
};

}  // namespace

__global__ __launch_bounds__(kEncBlock) void k_encode(EncodeArgs a) {
    extern __shared__ uint64_t s_dyn_enc[];
    uint64_t *s_tbl = s_dyn_enc;
    uint16_t *s_stage = reinterpret_cast<uint16_t *>(s_dyn_enc + a.tbl_n);
    __shared__ uint32_t s_tile;
    __shared__ uint64_t s_base;
    __shared__ uint32_t s_part[kEncBlock / kWave];

    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int wave = tid / kWave;
    const uint32_t S = a.chunk_syms;
    const uint32_t pitch = S + kEncPad;                 // u16 units
    const uint32_t nbins = a.nbins;

    for (uint32_t i = tid; i < a.tbl_n; i += kEncBlock) s_tbl[i] = a.enc[a.tbl_lo + i];
    TableView tbl{s_tbl, a.enc, a.tbl_lo, a.tbl_n};

    uint32_t *payload;
    uint64_t cap_words;
    if (a.container) {
        const uint64_t off = a.ctl->off_payload;
        payload = reinterpret_cast<uint32_t *>(a.container + off);
        cap_words = (a.capacity >= off) ? (a.capacity - off) / 4u : 0u;
    } else {
        payload = a.payload;
        cap_words = a.payload_cap_words;
    }

    if (tid == 0) s_tile = atomicAdd(&a.ctl->ticket_e, 1u);
    __syncthreads();
    uint32_t tile = s_tile;
    uint16_t *my_wave_stage = s_stage + (uint32_t)wave * kWave * pitch;
    const uint16_t *my_stage = my_wave_stage + (uint32_t)lane * pitch;

    while (tile < a.n_tiles) {
        uint32_t next_tile = 0;
        if (tid == 0) next_tile = atomicAdd(&a.ctl->ticket_e, 1u);

        // ---- stage this wavefront's 64 chunks ----
        const uint64_t chunk0 = (uint64_t)tile * kEncBlock + (uint64_t)wave * kWave;
        const uint64_t sym_base = chunk0 * S;
        const uint32_t pieces = 8u * S;                  // 16-byte pieces per wavefront (64 * S / 8)
        for (uint32_t p = lane; p < pieces; p += kWave) {
            const uint64_t sym0 = sym_base + 8ull * p;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (sym0 + 8u <= a.n) v = *reinterpret_cast<const uint4 *>(a.codes + sym0);
            else if (sym0 < a.n) {
                uint32_t w[4] = {0, 0, 0, 0};
                for (uint32_t j = 0; j < 8u && sym0 + j < a.n; ++j) w[j >> 1] |= (uint32_t)a.codes[sym0 + j] << (16u * (j & 1u));
                v = make_uint4(w[0], w[1], w[2], w[3]);
            }
            const uint32_t cl = (8u * p) >> a.log2_chunk;
            const uint32_t within = (8u * p) & (S - 1u);
            *reinterpret_cast<uint4 *>(my_wave_stage + cl * pitch + within) = v;
        }
        __syncthreads();

        // ---- pass A: bits of my chunk ----
        const uint64_t c = chunk0 + lane;
        uint32_t nsym = 0;
        if (c * S < a.n) { const uint64_t rem = a.n - c * S; nsym = rem < S ? (uint32_t)rem : S; }
        uint32_t bits = 0;
        for (uint32_t k = 0; k < S; k += 8) {
            const uint4 v = *reinterpret_cast<const uint4 *>(my_stage + k);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (uint32_t j = 0; j < 8; ++j) {
                uint32_t code = (w[j >> 1] >> (16u * (j & 1u))) & 0xffffu;
                if (code >= nbins) code = 0;
                const uint32_t L = tbl.length(code);
                bits += (k + j < nsym) ? L : 0u;
            }
        }
        const uint32_t words = (bits + 31u) / 32u;
        uint32_t tile_words;
        const uint32_t excl = block_excl_scan<uint32_t, kEncBlock / kWave>(words, s_part, tile_words);
        if (wave == 0) {
            const uint64_t base = chained_scan_wave(a.desc, tile, tile_words, &a.ctl->status);
            if (lane == 0) {
                s_base = base;
                if (tile + 1 == a.n_tiles) a.ctl->payload_words = base + tile_words;
            }
        }
        __syncthreads();
        const uint64_t off = s_base + excl;
        if (c < a.n_chunks) {
            if (off > 0xffffffffull) atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);
            a.chunk_off[c] = (uint32_t)off;
        }

        // ---- pass B: pack and write ----
        if (nsym) {
            uint64_t buf = 0;
            uint32_t nb = 0;
            uint64_t wpos = off;
            bool overflow = false;
            auto emit = [&](uint32_t word) {
                if (wpos < cap_words) payload[wpos] = word;
                else overflow = true;
                ++wpos;
            };
            auto put = [&](uint64_t bitsv, uint32_t L) {   // 1 <= L <= 32, nb <= 31
                buf |= bitsv << (64u - nb - L);
                nb += L;
                if (nb >= 32u) { emit((uint32_t)(buf >> 32)); buf <<= 32; nb -= 32u; }
            };
            for (uint32_t k = 0; k < S; k += 8) {
                const uint4 v = *reinterpret_cast<const uint4 *>(my_stage + k);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (uint32_t j = 0; j < 8; ++j) {
                    if (k + j < nsym) {
                        uint32_t code = (w[j >> 1] >> (16u * (j & 1u))) & 0xffffu;
                        if (code >= nbins) code = 0;
                        const uint64_t e = tbl.full(code);
                        const uint32_t L = (uint32_t)(e & 63u);
                        const uint64_t cw = e >> 6;
                        if (L > 32u) { put(cw >> 32, L - 32u); put(cw & 0xffffffffull, 32u); }
                        else if (L) put(cw, L);
                    }
                }
            }
            if (nb) emit((uint32_t)(buf >> 32));
            if (overflow) atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);
        }

        if (tid == 0) s_tile = next_tile;
        __syncthreads();
        tile = s_tile;
    }

    // ---- the last workgroup to finish seals the container ----
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t prev = atomicAdd(&a.ctl->done_e, 1u);
        if (prev == gridDim.x - 1u) {
            __threadfence();
            const uint64_t pw = __hip_atomic_load(&a.ctl->payload_words, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t st = __hip_atomic_load(&a.ctl->status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (a.container) {
                Header *h = reinterpret_cast<Header *>(a.container);
                const uint64_t total = a.ctl->off_payload + 4ull * pw;
                h->payload_words = pw;
                h->total_bytes = total;
                h->status = st ? 1u : 0u;
                a.ctl->total_bytes = total;
            }
            if (a.payload_words_out) *a.payload_words_out = pw;
        }
    }
}

}  // namespace comet
