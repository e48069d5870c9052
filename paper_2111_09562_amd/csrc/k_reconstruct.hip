// Fused decompression kernel (COMET Sec. 3.4 / Sec. 4.1 run backwards):
// chunk-parallel Huffman decode -> outlier patch -> plane-wise 2-D inclusive
// prefix sums (Lorenzo reconstruction) -> dequantise -> verbatim values ->
// re-zero filter -> coalesced fp32 store.  Codes never travel through global
// memory: a strip of whole rows is decoded straight into LDS, scanned there and
// written out once.
//
// Work unit: a group of whole planes when a plane is small, or one plane cut
// into strips of rows (column sums carried in LDS from strip to strip) when it
// is large.  One lane decodes one chunk; LDS rows have an odd pitch so that
// both the per-row and the per-column sweeps are bank-conflict free.
#include "comet_kernels.h"

namespace comet {

namespace {

struct BitReader {
    const uint32_t *p, *end;
    uint64_t buf;      // next bits, left aligned; at least 33 valid after every symbol
    uint32_t nb;       // valid bits in buf
    uint32_t nw;       // the word after buf, already loaded
    __device__ inline static uint32_t ldw(const uint32_t *q, const uint32_t *e) { return q < e ? *q : 0u; }
    __device__ inline void init(const uint32_t *begin, const uint32_t *e) {
        end = e;
        buf = ((uint64_t)ldw(begin, e) << 32) | ldw(begin + 1, e);
        nw = ldw(begin + 2, e);
        p = begin + 3;
        nb = 64;
    }
    __device__ inline void consume(uint32_t L) {
        if (L < nb) { buf <<= L; nb -= L; }
        else {                      // a long code that runs into the look-ahead word
            const uint32_t extra = L - nb;
            buf = ((uint64_t)nw << 32) << extra;
            nb = 32u - extra;
            nw = ldw(p, end); ++p;
        }
        if (nb <= 32u) { buf |= (uint64_t)nw << (32u - nb); nb += 32u; nw = ldw(p, end); ++p; }
    }
};

struct LdsTables {
    const uint32_t *lut;
    const uint64_t *limit, *first;
    const uint32_t *findex;
    const uint16_t *sorted;
    uint32_t max_len, n_active;
    int32_t radius;
};

__device__ inline uint32_t decode_symbol(BitReader &br, const LdsTables &t) {
    const uint32_t e = t.lut[br.buf >> (64 - kLutBits)];
    uint32_t L, sym;
    if (e & 0xffu) {
        L = e & 0xffu;
        const int32_t d = (int32_t)e >> 8;                  // the table holds residuals
        sym = (d == -32768) ? 0u : (uint32_t)(d + t.radius);
    } else {
        const uint64_t win = br.buf | ((uint64_t)br.nw >> (br.nb - 32u));
        L = e >> 8;                                         // the shortest length this prefix can have
        if (L <= (uint32_t)kLutBits) L = kLutBits + 1;
        while (L < t.max_len && win >= t.limit[L]) ++L;
        if (L > 57u) L = 57u;
        uint64_t idx = t.findex[L] + ((win >> (64u - L)) - t.first[L]);
        if (idx >= t.n_active) idx = t.n_active - 1u;      // only reachable with a corrupt stream
        sym = t.sorted[idx];
    }
    br.consume(L);
    return sym;
}

__device__ inline void load_tables(const DecodeTables &g, uint32_t *s_lut, uint64_t *s_limit, uint64_t *s_first,
                                   uint32_t *s_findex, LdsTables &t) {
    for (uint32_t i = threadIdx.x; i < kLutSize; i += blockDim.x) s_lut[i] = g.lut[i];
    for (uint32_t i = threadIdx.x; i < 65u; i += blockDim.x) { s_limit[i] = g.limit[i]; s_first[i] = g.first_code[i]; s_findex[i] = g.first_index[i]; }
    t.lut = s_lut; t.limit = s_limit; t.first = s_first; t.findex = s_findex; t.sorted = g.sorted;
    t.max_len = g.meta[0]; t.n_active = g.meta[1]; t.radius = (int32_t)g.meta[3];
}

// first record index whose key is >= target; all 64 lanes of one wavefront take
// part (65-ary search: a handful of dependent loads instead of ~20)
__device__ inline uint64_t record_lower_bound(const uint32_t *rec, uint64_t n_rec, uint32_t target) {
    uint64_t lo = 0, hi = n_rec;
    const int lane = lane_id();
    while (lo < hi) {
        const uint64_t span = hi - lo;
        const uint64_t step = (span + 64u) / 65u;
        const uint64_t p = lo + (uint64_t)(lane + 1) * step - 1u;
        const bool less = (p < hi) ? (rec[2 * p] < target) : false;
        const int c = __popcll(__ballot(less));
        const uint64_t pc = lo + (uint64_t)(c + 1) * step - 1u;
        const uint64_t new_hi = (c < kWave && pc < hi) ? pc : hi;
        lo = lo + (uint64_t)c * step;
        hi = new_hi;
    }
    return lo;
}

}  // namespace

template <int MODE>
__global__ __launch_bounds__(kDecBlock) void k_reconstruct(ReconArgs a) {
    extern __shared__ int32_t s_dyn_rec[];          // tile, then the column carry
    __shared__ uint32_t s_lut[kLutSize];
    __shared__ uint64_t s_limit[65];
    __shared__ uint64_t s_first[65];
    __shared__ uint32_t s_findex[65];

    if (MODE == 0 && (a.ctl->status & ST_FORMAT)) return;
    // launched behind the kernel for chunks of 64 symbols: only containers that one has left alone
    if (MODE == 0 && a.skip_chunk64 && reinterpret_cast<const Header *>(a.container)->chunk_syms == 64u) return;

    const int tid = threadIdx.x;
    int32_t *tile = s_dyn_rec;
    int32_t *carry = s_dyn_rec + (size_t)a.tile_rows * a.pitch;

    // ---- where the pieces are ----
    const uint32_t *chunk_off = a.chunk_off, *payload = a.payload, *rec = a.rec;
    uint64_t payload_words = a.payload_words, n_rec = a.n_rec;
    uint32_t S = a.chunk_syms, n_chunks = a.n_chunks;
    int32_t radius = a.radius;
    float eb = a.eb, ebx2 = a.ebx2;
    bool zero_chunks = false;
    LdsTables t{};
    if (MODE == 0) {
        const Header *h = reinterpret_cast<const Header *>(a.container);
        zero_chunks = h->version == 2u;
        chunk_off = reinterpret_cast<const uint32_t *>(a.container + h->off_chunk);
        rec = reinterpret_cast<const uint32_t *>(a.container + h->off_outlier);
        payload = reinterpret_cast<const uint32_t *>(a.container + h->off_payload);
        payload_words = h->payload_words;
        n_rec = h->n_rec;
        S = h->chunk_syms;
        n_chunks = h->n_chunks;
        radius = (int32_t)(h->nbins / 2u);
        eb = __uint_as_float(h->eb_bits);
        ebx2 = __uint_as_float(h->ebx2_bits);
        load_tables(a.t, s_lut, s_limit, s_first, s_findex, t);
        __syncthreads();
    }
    const uint32_t W = a.W, H = a.H, pitch = a.pitch;
    const uint32_t P = H * W;
    const uint32_t n = (uint32_t)a.n;

    for (uint32_t unit = blockIdx.x; unit < a.n_units; unit += gridDim.x) {
        uint32_t e_begin, unit_rows, planes_here;
        if (a.use_carry) { e_begin = unit * P; unit_rows = H; planes_here = 1; }
        else {
            const uint32_t p0 = unit * a.planes_per_unit;
            planes_here = a.planes - p0 < a.planes_per_unit ? a.planes - p0 : a.planes_per_unit;
            e_begin = p0 * P;
            unit_rows = planes_here * H;
        }
        uint64_t rpos = 0;
        if (n_rec) rpos = record_lower_bound(rec, n_rec, 2u * e_begin);
        if (a.use_carry) for (uint32_t w = tid; w < W; w += kDecBlock) carry[w] = 0;

        for (uint32_t row0 = 0; row0 < unit_rows; row0 += a.tile_rows) {
            const uint32_t rows = unit_rows - row0 < a.tile_rows ? unit_rows - row0 : a.tile_rows;
            const uint32_t e0 = e_begin + row0 * W;
            const uint32_t ne = rows * W;
            const uint32_t e1 = e0 + ne;

            // ---- 1. residuals into the tile ----
            if (MODE == 0) {
                const uint32_t c_lo = e0 / S;
                const uint32_t c_hi = (e1 - 1u) / S + 1u;
                for (uint32_t c = c_lo + tid; c < c_hi && c < n_chunks; c += kDecBlock) {
                    uint64_t w0 = chunk_off[c];
                    uint64_t w1 = (c + 1u < n_chunks) ? chunk_off[c + 1u] : payload_words;
                    if (w1 > payload_words) w1 = payload_words;
                    if (w0 > w1) w0 = w1;
                    const bool no_words = zero_chunks && w0 == w1;        // container version 2: the centre code throughout
                    BitReader br;
                    br.init(payload + w0, payload + w1);
                    const uint64_t s0 = (uint64_t)c * S;
                    uint32_t nsym = (n - s0 < S) ? (uint32_t)(n - s0) : S;
                    if (s0 + nsym > e1) nsym = (uint32_t)(e1 - s0);       // nothing past the strip is needed
                    uint32_t k = 0;
                    if (no_words) k = s0 < e0 ? (uint32_t)(e0 - s0) : 0u;
                    for (; s0 + k < e0; ++k) (void)decode_symbol(br, t);  // symbols that belong to the previous strip
                    const uint32_t l0 = (uint32_t)(s0 + k - e0);
                    uint32_t row = fdiv(l0, a.divW);
                    uint32_t col = l0 - row * W;
                    int32_t *dst = tile + row * pitch;
                    for (; k < nsym; ++k) {
                        const uint32_t sym = no_words ? (uint32_t)radius : decode_symbol(br, t);
                        dst[col] = sym ? (int32_t)sym - radius : 0;
                        if (++col == W) { col = 0; dst += pitch; }
                    }
                }
            } else {
                uint32_t row = fdiv((uint32_t)tid, a.divW);
                uint32_t col = (uint32_t)tid - row * W;
                const uint32_t drow = fdiv((uint32_t)kDecBlock, a.divW);
                const uint32_t dcol = (uint32_t)kDecBlock - drow * W;
                for (uint32_t l = tid; l < ne; l += kDecBlock) {
                    const uint32_t sym = a.codes_in[e0 + l];
                    tile[row * pitch + col] = sym ? (int32_t)sym - radius : 0;
                    row += drow; col += dcol;
                    if (col >= W) { col -= W; ++row; }
                }
            }
            __syncthreads();

            // ---- 2. escaped residuals from the outlier list ----
            uint64_t rec_begin = rpos, rec_end = rpos;
            if (n_rec) {
                uint32_t mine = 0;
                for (uint64_t k = rpos + tid; k < n_rec; k += kDecBlock) {
                    const uint32_t key = rec[2 * k];
                    if (key >= 2u * e1) break;
                    ++mine;
                    if (!(key & 1u)) {
                        const uint32_t l = (key >> 1) - e0;
                        const uint32_t row = fdiv(l, a.divW);
                        if (l < ne) tile[row * pitch + (l - row * W)] = (int32_t)rec[2 * k + 1];
                    }
                }
                rec_end = rpos + wave_sum<uint32_t>(mine);
                rpos = rec_end;
                __syncthreads();
            }

            // ---- 3. prefix sums along W, one lane per row ----
            for (uint32_t r = tid; r < rows; r += kDecBlock) {
                int32_t *p = tile + r * pitch;
                uint32_t acc = 0;
                for (uint32_t k = 0; k < W; ++k) { acc += (uint32_t)p[k]; p[k] = (int32_t)acc; }
            }
            __syncthreads();

            // ---- 4. prefix sums along H, dequantise, re-zero; one lane per column ----
            if (a.use_carry) {
                for (uint32_t w = tid; w < W; w += kDecBlock) {
                    uint32_t acc = (uint32_t)carry[w];
                    int32_t *p = tile + w;
                    for (uint32_t h = 0; h < rows; ++h, p += pitch) {
                        acc += (uint32_t)*p;
                        float v = (float)(int32_t)acc * ebx2;
                        if (fabsf(v) <= eb) v = 0.0f;
                        *p = __float_as_int(v);
                    }
                    carry[w] = (int32_t)acc;
                }
            } else {
                const uint32_t ncols = planes_here * W;
                for (uint32_t cidx = tid; cidx < ncols; cidx += kDecBlock) {
                    const uint32_t g = fdiv(cidx, a.divW);
                    const uint32_t w = cidx - g * W;
                    int32_t *p = tile + (size_t)g * H * pitch + w;
                    uint32_t acc = 0;
                    for (uint32_t h = 0; h < H; ++h, p += pitch) {
                        acc += (uint32_t)*p;
                        float v = (float)(int32_t)acc * ebx2;
                        if (fabsf(v) <= eb) v = 0.0f;
                        *p = __float_as_int(v);
                    }
                }
            }
            __syncthreads();

            // ---- 5. verbatim values ----
            if (rec_end > rec_begin) {
                for (uint64_t k = rec_begin + tid; k < rec_end; k += kDecBlock) {
                    const uint32_t key = rec[2 * k];
                    if (key & 1u) {
                        const uint32_t l = (key >> 1) - e0;
                        const uint32_t row = fdiv(l, a.divW);
                        float v = __uint_as_float(rec[2 * k + 1]);
                        if (fabsf(v) <= eb) v = 0.0f;
                        if (l < ne) tile[row * pitch + (l - row * W)] = __float_as_int(v);
                    }
                }
                __syncthreads();
            }

            // ---- 6. coalesced store ----
            {
                uint32_t row = fdiv((uint32_t)tid, a.divW);
                uint32_t col = (uint32_t)tid - row * W;
                const uint32_t drow = fdiv((uint32_t)kDecBlock, a.divW);
                const uint32_t dcol = (uint32_t)kDecBlock - drow * W;
                for (uint32_t l = tid; l < ne; l += kDecBlock) {
                    a.out[e0 + l] = __int_as_float(tile[row * pitch + col]);
                    row += drow; col += dcol;
                    if (col >= W) { col -= W; ++row; }
                }
            }
            __syncthreads();
        }
    }
}

template __global__ void k_reconstruct<0>(ReconArgs);
template __global__ void k_reconstruct<1>(ReconArgs);

// Stage entry point: decode only, codes to global memory (one lane per chunk).
__global__ __launch_bounds__(kDecBlock) void k_decode_only(ReconArgs a) {
    __shared__ uint32_t s_lut[kLutSize];
    __shared__ uint64_t s_limit[65];
    __shared__ uint64_t s_first[65];
    __shared__ uint32_t s_findex[65];
    if (a.ctl->status & ST_FORMAT) return;
    LdsTables t{};
    load_tables(a.t, s_lut, s_limit, s_first, s_findex, t);
    __syncthreads();
    const uint32_t S = a.chunk_syms;
    for (uint64_t c = (uint64_t)blockIdx.x * kDecBlock + threadIdx.x; c < a.n_chunks; c += (uint64_t)gridDim.x * kDecBlock) {
        uint64_t w0 = a.chunk_off[c];
        uint64_t w1 = (c + 1u < a.n_chunks) ? a.chunk_off[c + 1u] : a.payload_words;
        if (w1 > a.payload_words) w1 = a.payload_words;
        if (w0 > w1) w0 = w1;
        const bool no_words = a.zero_chunks && w0 == w1;        // container version 2: the centre code throughout
        BitReader br;
        br.init(a.payload + w0, a.payload + w1);
        const uint64_t s0 = c * S;
        const uint32_t nsym = (a.n - s0 < S) ? (uint32_t)(a.n - s0) : S;
        for (uint32_t k = 0; k < nsym; ++k) a.codes_out[s0 + k] = no_words ? (uint16_t)t.radius : (uint16_t)decode_symbol(br, t);
    }
}

}  // namespace comet
