// Quantise kernel: prequantisation, 2-D Lorenzo prediction, quantisation codes,
// histogram and outlier records in one sweep over the input (COMET Sec. 4.1,
// first three steps of the modified cuSZ pipeline; Sec. 2.2 for the bound).
//
// Layout of the work: the tensor is cut into flat tiles of kTile consecutive
// elements (NCHW linear order).  A workgroup takes tiles by ticket, keeps its 16
// elements per lane in registers, and gets the three Lorenzo neighbours of an
// element by re-reading the *input* one row back (the prequantised value is a
// pure function of the input, so no tile depends on another one).  Outlier
// records are placed in ascending index order with a chained scan over tiles.
// The histogram is privatised in LDS (a window of bins around the centre bin
// when nbins is large) and flushed once per workgroup.
#include "comet_kernels.h"

namespace comet {

namespace {

constexpr int kVec = 4;
constexpr int kIter = kQuantTile / (kQuantBlock * kVec);
static_assert(kIter * kQuantBlock * kVec == kQuantTile, "tile shape");

__device__ inline int32_t prequant(float x, float r) {
    const float t = x * r;
    return (fabsf(t) < 16777216.0f) ? (int32_t)rintf(t) : 0;
}

// true if the element must be stored verbatim: its lattice value, as the
// decompressor will compute it, misses the bound (judged in fp64), or it has no
// lattice value at all.
__device__ inline bool needs_verbatim(float x, int32_t q, float r, float ebx2, float eb) {
    const float t = x * r;
    if (!(fabsf(t) < 16777216.0f)) return true;
    const float y = (float)q * ebx2;
    return !(fabs((double)x - (double)y) <= (double)eb);
}

}  // namespace

__global__ __launch_bounds__(kQuantBlock) void k_quantize(QuantArgs a) {
    extern __shared__ uint32_t s_hist[];            // a.win_n bins
    __shared__ uint32_t s_tile;
    __shared__ uint64_t s_base;
    __shared__ uint64_t s_part64[kQuantBlock / kWave];
    __shared__ uint32_t s_part32[kQuantBlock / kWave];

    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int wave = tid / kWave;

    for (uint32_t i = tid; i < a.win_n; i += kQuantBlock) s_hist[i] = 0;
    if (tid == 0) s_tile = atomicAdd(&a.ctl->ticket_q, 1u);
    __syncthreads();
    uint32_t tile = s_tile;

    uint32_t centre_count = 0;       // hits of the centre bin (residual 0), kept out of the LDS atomics
    uint32_t nnz_local = 0;
    uint32_t vrec_local = 0;
    const uint32_t n = (uint32_t)a.n;
    const uint32_t W = a.divW.d;
    const uint32_t H = a.divH.d;
    const int32_t radius = a.radius;

    while (tile < a.n_tiles) {
        uint32_t next_tile = 0;
        if (tid == 0) next_tile = atomicAdd(&a.ctl->ticket_q, 1u);   // latency hidden behind the tile

        const uint32_t start = tile * (uint32_t)kQuantTile;
        int32_t dres[kIter][kVec];
        uint32_t flags[kIter];          // bit j: escape code, bit 4+j: verbatim
        uint32_t counts = 0;            // four 8-bit record counts, one per iteration

#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            flags[it] = 0;
            const uint32_t i0 = start + (uint32_t)it * (kQuantBlock * kVec) + (uint32_t)tid * kVec;
            if (i0 >= n) continue;
            const uint32_t nvalid = (n - i0 >= (uint32_t)kVec) ? (uint32_t)kVec : (n - i0);
            float xv[kVec];
            if (nvalid == kVec) {
                const float4 v = *reinterpret_cast<const float4 *>(a.x + i0);
                xv[0] = v.x; xv[1] = v.y; xv[2] = v.z; xv[3] = v.w;
            } else {
#pragma unroll
                for (int j = 0; j < kVec; ++j) xv[j] = ((uint32_t)j < nvalid) ? a.x[i0 + j] : 0.0f;
            }
            // position of the first element inside its plane
            const uint32_t row0 = fdiv(i0, a.divW);
            uint32_t w = i0 - row0 * W;
            uint32_t h = row0 - fdiv(row0, a.divH) * H;
            // the row above: x[i0-W-1 .. i0-W+3]; left neighbour: x[i0-1].  Indices that
            // would be negative are never used (they belong to h == 0 or w == 0).
            float xu[kVec + 1];
#pragma unroll
            for (int k = 0; k < kVec + 1; ++k) {
                const int64_t idx = (int64_t)i0 - (int64_t)W - 1 + k;
                xu[k] = a.x[idx > 0 ? idx : 0];
            }
            const float xl = a.x[i0 > 0 ? i0 - 1 : 0];
            int32_t qu[kVec + 1];
#pragma unroll
            for (int k = 0; k < kVec + 1; ++k) qu[k] = prequant(xu[k], a.r);
            int32_t qprev = prequant(xl, a.r);
            uint16_t code[kVec];
            uint32_t f = 0;
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                const int32_t q = prequant(xv[j], a.r);
                const uint32_t left = (w > 0) ? (uint32_t)qprev : 0u;
                const uint32_t up = (h > 0) ? (uint32_t)qu[j + 1] : 0u;
                const uint32_t upleft = (h > 0 && w > 0) ? (uint32_t)qu[j] : 0u;
                const int32_t d = (int32_t)((uint32_t)q - left - up + upleft);
                dres[it][j] = d;
                qprev = q;
                uint32_t c;
                if (d > -radius && d < radius) c = (uint32_t)(d + radius);
                else { c = 0; if ((uint32_t)j < nvalid) f |= 1u << j; }
                code[j] = (uint16_t)c;
                if ((uint32_t)j < nvalid) {
                    if (needs_verbatim(xv[j], q, a.r, a.ebx2, a.eb)) f |= 16u << j;
                    nnz_local += (xv[j] != 0.0f) ? 1u : 0u;
                    if (c == (uint32_t)radius) ++centre_count;
                    else {
                        const uint32_t bin = c - a.win_lo;
                        if (bin < a.win_n) atomicAdd(&s_hist[bin], 1u);
                        else atomicAdd(&a.hist[c], 1u);
                    }
                }
                if (++w == W) { w = 0; if (++h == H) h = 0; }
            }
            flags[it] = f;
            counts |= (uint32_t)__popc(f) << (8 * it);
            if (nvalid == kVec) {
                uint2 pk;
                pk.x = (uint32_t)code[0] | ((uint32_t)code[1] << 16);
                pk.y = (uint32_t)code[2] | ((uint32_t)code[3] << 16);
                *reinterpret_cast<uint2 *>(a.codes + i0) = pk;
            } else {
#pragma unroll
                for (int j = 0; j < kVec; ++j) if ((uint32_t)j < nvalid) a.codes[i0 + j] = code[j];
            }
        }

        // ---- outlier records: ascending index = iteration-major, lane-major ----
        const int any = __syncthreads_or(counts != 0u);
        uint64_t excl4 = 0, tot4 = 0;
        if (any) {
            // four 16-bit lanes of one 64-bit scan: per-iteration exclusive ranks
            uint64_t packed = 0;
#pragma unroll
            for (int it = 0; it < kIter; ++it) packed |= (uint64_t)((counts >> (8 * it)) & 0xffu) << (16 * it);
            excl4 = block_excl_scan<uint64_t, kQuantBlock / kWave>(packed, s_part64, tot4);
        }
        uint64_t tile_total = 0;
#pragma unroll
        for (int it = 0; it < kIter; ++it) tile_total += (tot4 >> (16 * it)) & 0xffffu;
        if (wave == 0) {
            const uint64_t base = chained_scan_wave(a.desc, tile, tile_total, &a.ctl->status);
            if (lane == 0) {
                s_base = base;
                if (tile + 1 == a.n_tiles) a.ctl->n_rec = base + tile_total;
            }
        }
        __syncthreads();
        if (any) {
            uint64_t pos_it = s_base;
#pragma unroll
            for (int it = 0; it < kIter; ++it) {
                uint64_t pos = pos_it + ((excl4 >> (16 * it)) & 0xffffu);
                pos_it += (tot4 >> (16 * it)) & 0xffffu;
                const uint32_t f = flags[it];
                if (!f) continue;
                const uint32_t i0 = start + (uint32_t)it * (kQuantBlock * kVec) + (uint32_t)tid * kVec;
#pragma unroll
                for (int j = 0; j < kVec; ++j) {
                    if (f & (1u << j)) {
                        if (pos < a.rec_cap) { uint2 rc; rc.x = 2u * (i0 + j); rc.y = (uint32_t)dres[it][j]; reinterpret_cast<uint2 *>(a.rec)[pos] = rc; }
                        else atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);
                        ++pos;
                    }
                    if (f & (16u << j)) {
                        if (pos < a.rec_cap) { uint2 rc; rc.x = 2u * (i0 + j) + 1u; rc.y = __float_as_uint(a.x[i0 + j]); reinterpret_cast<uint2 *>(a.rec)[pos] = rc; }
                        else atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);
                        ++pos;
                        ++vrec_local;
                    }
                }
            }
        }
        if (tid == 0) s_tile = next_tile;
        __syncthreads();
        tile = s_tile;
    }

    // ---- flush the private histogram and the counters ----
    {
        const uint32_t c = wave_sum<uint32_t>(centre_count);
        if (lane == 0 && c) {
            const uint32_t bin = (uint32_t)radius - a.win_lo;
            if (bin < a.win_n) atomicAdd(&s_hist[bin], c);
            else atomicAdd(&a.hist[radius], c);
        }
    }
    __syncthreads();
    for (uint32_t i = tid; i < a.win_n; i += kQuantBlock) {
        const uint32_t v = s_hist[i];
        if (v) atomicAdd(&a.hist[a.win_lo + i], v);
    }
    uint32_t tot;
    (void)block_excl_scan<uint32_t, kQuantBlock / kWave>(nnz_local, s_part32, tot);
    if (tid == 0 && tot) atomicAdd((unsigned long long *)&a.ctl->nnz, (unsigned long long)tot);
    (void)block_excl_scan<uint32_t, kQuantBlock / kWave>(vrec_local, s_part32, tot);
    if (tid == 0 && tot) atomicAdd((unsigned long long *)&a.ctl->n_vrec, (unsigned long long)tot);
}

}  // namespace comet
