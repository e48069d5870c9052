// Quantise kernel: prequantisation, 2-D Lorenzo prediction, quantisation codes,
// histogram and outlier records in one sweep over the input (COMET Sec. 4.1,
// first three steps of the modified cuSZ pipeline; Sec. 2.2 for the bound).
//
// Layout of the work: the tensor is cut into flat tiles of kQuantTile consecutive
// elements (NCHW linear order).  A workgroup takes tiles by ticket, keeps its 16
// elements per lane in registers, and gets the three Lorenzo neighbours of an
// element by re-reading the *input* one row back (the prequantised value is a
// pure function of the input, so no tile depends on another one).  Outlier
// records are placed in ascending index order with a chained scan over tiles.
// The histogram is privatised in LDS (a window of bins around the centre bin
// when nbins is large) and flushed once per workgroup.
//
// The kernel is bound by instruction issue, not by HBM, so interior tiles (every
// load in range, planes at least 4 wide) take a branch-free path: plane-boundary
// handling is two precomputed masks per lane, the error-bound check is a cheap
// fp32 filter that only falls back to the exact fp64 comparison for the rare
// element within a few ulp of the bound, and outlier bookkeeping is deferred to
// a slow path that runs only for tiles that have outliers.
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

template <bool FULLWIN>
__global__ __launch_bounds__(kQuantBlock) void k_quantize(QuantArgs a) {
    extern __shared__ uint32_t s_dyn_q[];           // histogram window (a.win_n bins), then the record buffer
    uint32_t *s_hist = s_dyn_q;
    uint2 *s_rec = reinterpret_cast<uint2 *>(s_dyn_q + a.win_n);
    __shared__ uint32_t s_seg;
    __shared__ uint64_t s_base;
    __shared__ uint64_t s_part64[kQuantBlock / kWave];
    __shared__ uint32_t s_part32[kQuantBlock / kWave];

    const int tid = threadIdx.x;
    const int lane = lane_id();

    const float *xin = static_cast<const float *>(a.x);      // this kernel takes fp32 only
    for (uint32_t i = tid; i < a.win_n; i += kQuantBlock) s_hist[i] = 0;
    // A workgroup owns one segment of consecutive tiles; segments are handed out by ticket so that
    // a segment is never started before the ones in front of it (the final offsets wait on them).
    if (tid == 0) s_seg = atomicAdd(&a.ctl->ticket_q, 1u);
    __syncthreads();
    const uint32_t seg = s_seg;
    const uint32_t tile_lo = seg * a.tiles_per_seg;
    const uint32_t tile_hi = (tile_lo + a.tiles_per_seg < a.n_tiles) ? tile_lo + a.tiles_per_seg : a.n_tiles;
    if (tile_lo >= a.n_tiles) return;                // uniform

    uint32_t centre_count = 0;       // hits of the centre bin (residual 0), kept out of the LDS atomics
    uint32_t nnz_local = 0;
    uint32_t vrec_local = 0;
    const uint32_t n = (uint32_t)a.n;
    const uint32_t W = a.divW.d;
    const uint32_t H = a.divH.d;
    const int32_t radius = a.radius;
    const uint32_t code_span = a.nbins - 1u;        // residual + radius - 1 must be below this
    // an fp32 error above eb_lo needs the exact comparison (the fp32 subtraction is within one rounding)
    const float eb_lo = a.eb * (1.0f - 0x1p-20f);

    uint32_t seg_records = 0;        // records of this segment so far (uniform)
    bool overflow = false;           // the LDS record buffer was too small: a second pass re-derives them

    // Residuals of one tile by the general rules (bounds, planes of any width); with side effects
    // (codes, histogram, counters) on the first pass only.
    auto tile_general = [&](uint32_t start, int32_t (&dres)[kIter][kVec], bool side_effects) {
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            const uint32_t i0 = start + (uint32_t)it * (kQuantBlock * kVec) + (uint32_t)tid * kVec;
#pragma unroll
            for (int j = 0; j < kVec; ++j) dres[it][j] = 0;
            if (i0 >= n) continue;
            const uint32_t nvalid = (n - i0 >= (uint32_t)kVec) ? (uint32_t)kVec : (n - i0);
            float xv[kVec];
#pragma unroll
            for (int j = 0; j < kVec; ++j) xv[j] = ((uint32_t)j < nvalid) ? xin[i0 + j] : 0.0f;
            const uint32_t row0 = fdiv(i0, a.divW);
            uint32_t w = i0 - row0 * W;
            uint32_t h = row0 - fdiv(row0, a.divH) * H;
            // the row above: x[i0-W-1 .. i0-W+3]; left neighbour: x[i0-1].  Indices that
            // would be negative are never used (they belong to h == 0 or w == 0).
            float xu[kVec + 1];
#pragma unroll
            for (int k = 0; k < kVec + 1; ++k) {
                const int64_t idx = (int64_t)i0 - (int64_t)W - 1 + k;
                xu[k] = xin[idx > 0 ? idx : 0];
            }
            const float xl = xin[i0 > 0 ? i0 - 1 : 0];
            int32_t qu[kVec + 1];
#pragma unroll
            for (int k = 0; k < kVec + 1; ++k) qu[k] = prequant(xu[k], a.r);
            int32_t qprev = prequant(xl, a.r);
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                const int32_t q = prequant(xv[j], a.r);
                const uint32_t left = (w > 0) ? (uint32_t)qprev : 0u;
                const uint32_t upv = (h > 0) ? (uint32_t)qu[j + 1] : 0u;
                const uint32_t upleft = (h > 0 && w > 0) ? (uint32_t)qu[j] : 0u;
                const int32_t d = (int32_t)((uint32_t)q - left - upv + upleft);
                dres[it][j] = d;
                qprev = q;
                if (side_effects && (uint32_t)j < nvalid) {
                    const uint32_t c = (d > -radius && d < radius) ? (uint32_t)(d + radius) : 0u;
                    nnz_local += (xv[j] != 0.0f) ? 1u : 0u;
                    a.codes[i0 + j] = (uint16_t)c;
                    if (c == (uint32_t)radius) ++centre_count;
                    else {
                        const uint32_t bin = c - a.win_lo;
                        if (bin < a.win_n) atomicAdd(&s_hist[bin], 1u);
                        else atomicAdd(&a.hist[c], 1u);
                    }
                }
                if (++w == W) { w = 0; if (++h == H) h = 0; }
            }
        }
    };

    // Exact classification of a tile's elements and placement of its records, in ascending index
    // order (iteration-major, lane-major), at records [seg_records, ...) of the segment: into the
    // LDS buffer on the first pass, straight into the container (at `gbase`) on the second.
    auto tile_records = [&](uint32_t start, const int32_t (&dres)[kIter][kVec], bool to_global, uint64_t gbase) {
        uint32_t flags[kIter];          // bit j: escape code, bit 4+j: verbatim
        uint32_t counts = 0;            // four 8-bit record counts, one per iteration
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            const uint32_t i0 = start + (uint32_t)it * (kQuantBlock * kVec) + (uint32_t)tid * kVec;
            uint32_t f = 0;
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                if (i0 + (uint32_t)j < n) {
                    const int32_t d = dres[it][j];
                    if (!(d > -radius && d < radius)) f |= 1u << j;
                    const float x = xin[i0 + j];
                    if (needs_verbatim(x, prequant(x, a.r), a.r, a.ebx2, a.eb)) f |= 16u << j;
                }
            }
            flags[it] = f;
            counts |= (uint32_t)__popc(f) << (8 * it);
        }
        // four 16-bit lanes of one 64-bit scan: per-iteration exclusive ranks
        uint64_t packed = 0, tot4 = 0;
#pragma unroll
        for (int it = 0; it < kIter; ++it) packed |= (uint64_t)((counts >> (8 * it)) & 0xffu) << (16 * it);
        const uint64_t excl4 = block_excl_scan<uint64_t, kQuantBlock / kWave>(packed, s_part64, tot4);
        uint32_t pos_it = seg_records;
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            uint32_t pos = pos_it + (uint32_t)((excl4 >> (16 * it)) & 0xffffu);
            pos_it += (uint32_t)((tot4 >> (16 * it)) & 0xffffu);
            const uint32_t f = flags[it];
            if (!f) continue;
            const uint32_t i0 = start + (uint32_t)it * (kQuantBlock * kVec) + (uint32_t)tid * kVec;
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
#pragma unroll
                for (int type = 0; type < 2; ++type) {
                    if (!(f & ((type ? 16u : 1u) << j))) continue;
                    uint2 rc;
                    rc.x = 2u * (i0 + j) + (uint32_t)type;
                    rc.y = type ? __float_as_uint(xin[i0 + j]) : (uint32_t)dres[it][j];
                    if (to_global) {
                        if (gbase + pos < a.rec_cap) reinterpret_cast<uint2 *>(a.rec)[gbase + pos] = rc;
                        else atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);
                    } else if (pos < a.rec_lds) s_rec[pos] = rc;
                    if (type && !to_global) ++vrec_local;
                    ++pos;
                }
            }
        }
        seg_records = pos_it;
    };

    for (uint32_t tile = tile_lo; tile < tile_hi; ++tile) {
        const uint32_t start = tile * (uint32_t)kQuantTile;
        int32_t dres[kIter][kVec];
        bool any_flag = false;
        const bool interior = W >= (uint32_t)kVec && start >= W + 1u && start + (uint32_t)kQuantTile <= n;

        if (interior) {
            // ---------------- fast path: no bounds, no per-element branches ----------------
#pragma unroll
            for (int it = 0; it < kIter; ++it) {
                const uint32_t i0 = start + (uint32_t)it * (kQuantBlock * kVec) + (uint32_t)tid * kVec;
                const float4 v = *reinterpret_cast<const float4 *>(xin + i0);
                const float xv[kVec] = {v.x, v.y, v.z, v.w};
                const float *up = xin + (i0 - W - 1u);
                const float xu[kVec + 1] = {up[0], up[1], up[2], up[3], up[4]};
                const float xl = xin[i0 - 1u];
                // position of the first element inside its plane; wj = where the row wraps inside my four
                const uint32_t row0 = fdiv(i0, a.divW);
                const uint32_t w0 = i0 - row0 * W;
                const uint32_t h0 = row0 - fdiv(row0, a.divH) * H;
                const uint32_t wj = W - w0;                                   // 1 .. W
                const uint32_t h1 = (h0 + 1u == H) ? 0u : h0 + 1u;
                const uint32_t um0 = h0 ? ~0u : 0u, um1 = h1 ? ~0u : 0u;      // "has a row above" before / after the wrap
                int32_t qu[kVec + 1];
#pragma unroll
                for (int k = 0; k < kVec + 1; ++k) qu[k] = prequant(xu[k], a.r);
                int32_t qprev = prequant(xl, a.r);
                uint32_t code[kVec];
#pragma unroll
                for (int j = 0; j < kVec; ++j) {
                    const float t = xv[j] * a.r;
                    const int32_t q = (fabsf(t) < 16777216.0f) ? (int32_t)rintf(t) : 0;
                    const uint32_t lm = (j == 0) ? (w0 ? ~0u : 0u) : (((uint32_t)j != wj) ? ~0u : 0u);
                    const uint32_t um = ((uint32_t)j < wj) ? um0 : um1;
                    const uint32_t d = (uint32_t)q - ((uint32_t)qprev & lm) - ((uint32_t)qu[j + 1] & um) + ((uint32_t)qu[j] & lm & um);
                    dres[it][j] = (int32_t)d;
                    qprev = q;
                    const uint32_t c = d + (uint32_t)radius;
                    const bool inrange = (c - 1u) < code_span;
                    code[j] = inrange ? c : 0u;
                    // error-bound filter: |x - y| in fp32 is within one rounding of the exact error
                    const float err = fabsf(xv[j] - (float)q * a.ebx2);
                    const bool suspicious = !(err <= eb_lo);                  // also true for NaN / Inf / huge inputs
                    any_flag |= (!inrange) | suspicious;
                    nnz_local += (xv[j] != 0.0f) ? 1u : 0u;
                    if (code[j] == (uint32_t)radius) ++centre_count;
                    else if (FULLWIN) atomicAdd(&s_hist[code[j]], 1u);
                    else {
                        const uint32_t bin = code[j] - a.win_lo;
                        if (bin < a.win_n) atomicAdd(&s_hist[bin], 1u);
                        else atomicAdd(&a.hist[code[j]], 1u);
                    }
                }
                uint2 pk;
                pk.x = code[0] | (code[1] << 16);
                pk.y = code[2] | (code[3] << 16);
                *reinterpret_cast<uint2 *>(a.codes + i0) = pk;
            }
        } else {
            tile_general(start, dres, true);
            any_flag = true;                      // edge tiles are rare: let the exact classification decide
        }
        if (__syncthreads_or(any_flag ? 1 : 0)) {
            tile_records(start, dres, false, 0);
            if (seg_records > a.rec_lds) overflow = true;
        }
    }

    // ---- where this segment's records go: the sum of the counts of all segments in front ----
    // Every workgroup publishes its count once and adds up the counts in front of it; nobody waits
    // for anybody else's sum, only for counts, and those are published by workgroups that took their
    // ticket earlier and wait for nothing themselves.
    if (tid == 0) desc_store(&a.desc[seg], kDescAgg | (uint64_t)seg_records);
    {
        uint64_t sum = 0;
        bool failed = false;
        for (uint32_t idx = tid; idx < seg; idx += kQuantBlock) {
            uint64_t v = 0;
            uint32_t spins = 0;
            do {
                v = desc_load(&a.desc[idx]);
                if ((v >> 62) != 0) break;
                __builtin_amdgcn_s_sleep(1);
            } while (++spins < (1u << 22));
            if ((v >> 62) == 0) failed = true;
            sum += v & kDescMask;
        }
        if (failed) atomicOr(&a.ctl->status, (uint32_t)ST_INTERNAL);
        uint64_t total;
        (void)block_excl_scan<uint64_t, kQuantBlock / kWave>(sum, s_part64, total);
        if (tid == 0) {
            s_base = total;
            if (tile_hi == a.n_tiles) a.ctl->n_rec = total + seg_records;
        }
    }
    __syncthreads();
    const uint64_t base = s_base;
    if (seg_records) {
        if (!overflow) {
            for (uint32_t i = tid; i < seg_records; i += kQuantBlock) {
                if (base + i < a.rec_cap) reinterpret_cast<uint2 *>(a.rec)[base + i] = s_rec[i];
                else atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);
            }
        } else {
            // too many outliers for the LDS buffer: derive the records again, this time in place
            seg_records = 0;
            for (uint32_t tile = tile_lo; tile < tile_hi; ++tile) {
                const uint32_t start = tile * (uint32_t)kQuantTile;
                int32_t dres[kIter][kVec];
                tile_general(start, dres, false);
                tile_records(start, dres, true, base);
            }
        }
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

template __global__ void k_quantize<true>(QuantArgs);
template __global__ void k_quantize<false>(QuantArgs);

}  // namespace comet
