// Quantise kernels for planes up to 512 columns wide: prequantisation, 2-D Lorenzo
// prediction, quantisation codes, histogram and outlier records in one sweep over
// the input (COMET Sec. 4.1, first three steps of the modified cuSZ pipeline;
// Sec. 2.2 for the bound).
//
// The tensor is a matrix of planes*H rows of W floats.  A wavefront owns a run of
// consecutive rows and walks down it with lanes = columns (two adjacent columns per
// lane if W is even: one 8-byte load and one packed store of two codes), so every
// element is loaded and prequantised exactly once:
//   left neighbour      = the lane to the left (one DPP shift),
//   row above           = what the same lane held one step earlier (a register),
//   residual d          = rd - rd_above with rd = q - q_left (the row difference),
// and there is no index arithmetic per element.  Rows that take at most 32 lanes are
// walked K = 64 / lanes-per-row at a time (the row above then comes from the lanes of
// the row before through one cross-lane permute), so the 64 lanes still cover
// consecutive elements.  Loads and stores use buffer addressing: lanes without an
// element get an out-of-range offset, which the hardware ignores, so the loop is
// free of divergent branches and several steps of loads are kept in flight.
// The error-bound check is a cheap fp32 filter that falls back to the exact fp64
// comparison only for elements within a few ulp of the bound.
// The input may also be IEEE half or bfloat16: an element is widened to fp32 (exactly)
// as it is loaded, and everything after the load is the fp32 pipeline.
//
// Outlier records (escapes and verbatim values) must end up in the container in
// element order.  k_quantize_rows appends them, in order, to a staging area of
// its run (through a small LDS buffer, so that the main loop holds no global store
// the compiler cannot count) and leaves the count; k_gather_records, a second small
// kernel, adds up the counts in front of a run and moves its records to their final
// place (a run with more records than its staging area holds is swept again, this
// time writing in place).  The histogram goes the same way: LDS windows are added
// to one of several partial histograms, which k_gather_records adds up.  Nothing
// waits for anything inside a kernel.
//
// Compression with a given code book (the REUSE kernels) is a single pass over the input: the
// lengths are known, so a wavefront encodes its own codes instead of storing them.  It keeps
// them in a ring in LDS and, 256 at a time, packs them with the lane layout of the encode
// kernel into a work area of its run; a run is a whole number of chunks, so no chunk is shared
// between wavefronts.  k_place_payload moves the words of every run to their final place, which
// depends on the sizes of all runs in front of it and on the number of outlier records.
#include <type_traits>

#include "comet_kernels.h"
#include "comet_encode.h"

namespace comet {

namespace {

__device__ inline bool needs_verbatim_rows(float x, int32_t q, float r, float ebx2, float eb) {
    const float t = x * r;
    if (!(fabsf(t) < 16777216.0f)) return true;
    const float y = (float)q * ebx2;
    return !(fabs((double)x - (double)y) <= (double)eb);
}

// value of the lane to the left (lane 0 receives 0).  Callers combine the result with additions
// only: a subtraction whose shifted operand the compiler folds into the instruction came out with
// its operands exchanged on gfx950.
__device__ inline int32_t lane_left(int32_t v) {
    return __builtin_amdgcn_update_dpp(0, v, 0x138, 0xf, 0xf, true);   // wave_shr:1
}

__device__ inline __amdgpu_buffer_rsrc_t rows_rsrc(const void *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

constexpr uint32_t kOob = 0x80000000u;      // byte offset beyond every run
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Element type of the input: IN = 0 fp32, 1 IEEE half, 2 bfloat16.  A 16-bit input is widened to
// fp32 (exactly) as it is loaded; everything after the load is the fp32 pipeline.
template <int IN> __device__ inline float widen16(uint32_t h) {
    if (IN == 1) return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
    return __uint_as_float(h << 16);
}
template <int IN> __device__ inline float load_elem(const void *x, size_t i) {
    if (IN == 0) return static_cast<const float *>(x)[i];
    return widen16<IN>(static_cast<const unsigned short *>(x)[i]);
}

struct SweepCounts {
    uint32_t nnz_lane = 0;      // per lane: non-zero inputs
    uint32_t oow = 0;           // wavefront-uniform: codes outside the LDS window (counted in the global histogram)
    uint32_t vrec = 0;          // wavefront-uniform: verbatim records
    uint16_t *oow_list = nullptr;   // LDS, kQuantOowList entries of this wavefront: such codes on their way to the global histogram
    uint32_t oow_held = 0;      // wavefront-uniform: entries of the list in use
};

// One sweep of a wavefront over rows [row_lo, row_hi).  PASS 0: everything (codes, histogram,
// counters), records into rec_dst[0 .. rec_cap) (the rest is only counted); PASS 1: records only,
// and a record that does not fit raises ST_CAPACITY.  Returns the number of records of the run.
// VEC: adjacent columns per lane (1, or 2 for even W: one 8-byte load, one packed code store and
// one cross-lane shift per pair); NSEG: segments of 64 lanes per row (1, 2, 4, 8); MULTI: a row
// takes at most 32 lanes, K rows per step (NSEG == 1); FULLWIN: every histogram bin is in the LDS
// window.
// REUSE: code book reuse.  s_len (LDS, u8[nbins]) holds the code lengths the caller brought; a code
// whose length is 0 becomes an escape, there is no histogram, and an escape that the table has no
// code word for raises ST_CODEBOOK.  In PASS 0 the codes go to the ring of `enc` in LDS and are encoded
// from there (tbl: the encode table; FULLWIN then says that all of it is in LDS).
template <int VEC, int NSEG, bool MULTI, bool FULLWIN, int PASS, bool REUSE = false, int IN = 0>
__device__ inline uint32_t sweep_rows(const QuantArgs &a, uint32_t row_lo, uint32_t row_hi, uint32_t lane, uint32_t *s_hist,
                                      uint32_t hist_dummy, uint2 *s_buf, uint2 *rec_dst, uint64_t rec_cap, SweepCounts &cnt,
                                      const uint8_t *s_len = nullptr, RunEncoder *enc = nullptr,
                                      const TableView<FULLWIN> *tbl = nullptr) {
    const uint32_t W = a.divW.d, H = a.divH.d;
    const uint32_t LPR = W / (uint32_t)VEC;         // lanes per row
    const int32_t radius = a.radius;
    const uint32_t code_span = a.nbins - 1u;        // residual + radius - 1 must be below this
    // an fp32 error above eb_lo needs the exact comparison (the fp32 subtraction is within one rounding)
    const float eb_lo = a.eb * (1.0f - 0x1p-20f);
    const uint32_t hist_sub = lane & ((1u << a.hist_shift) - 1u);   // my copy of the histogram window

    const uint32_t e_lo = row_lo * W;
    const uint32_t n_el = (row_hi - row_lo) * W;
    constexpr uint32_t ES = IN ? 2u : 4u;                          // bytes per input element
    const __amdgpu_buffer_rsrc_t r_x = rows_rsrc(reinterpret_cast<const char *>(a.x) + (size_t)e_lo * ES, n_el * ES);
    const __amdgpu_buffer_rsrc_t r_c = rows_rsrc(a.codes + e_lo, n_el * 2u);
    const uint32_t K = MULTI ? a.rows_per_step : 1u;
    const uint32_t stride = MULTI ? K * W : W;                  // elements per step
    const uint32_t n_steps = (row_hi - row_lo + K - 1u) / K;
    uint32_t cur = 0;                                           // records so far (uniform)

    // lanes -> columns
    uint32_t col[NSEG];                                         // element offset of my first column inside a step, kOob / 4 if none
    uint32_t w0 = lane * VEC;                                   // MULTI: my first column
    bool first_col = false;                                     // MULTI: I hold column 0 of my row
    bool top_rows = false;                                      // MULTI: my row is the first one of a step
    uint32_t h_lane = 0;                                        // MULTI: my row inside its plane
    if (MULTI) {
        const uint32_t kr = fdiv(lane * VEC, a.divW);
        w0 = lane * VEC - kr * W;
        col[0] = (kr < K) ? lane * VEC : kOob / 4u;
        first_col = w0 == 0u;
        top_rows = lane < LPR;
        const uint32_t r0 = row_lo + kr;
        h_lane = r0 - fdiv(r0, a.divH) * H;
    } else {
#pragma unroll
        for (int s = 0; s < NSEG; ++s) {
            const uint32_t c = ((uint32_t)s * kWave + lane) * VEC;
            col[s] = (c < W) ? c : kOob / 4u;
        }
    }
    uint32_t h_row = row_lo - fdiv(row_lo, a.divH) * H;        // !MULTI: row of the current step inside its plane (uniform)
    const uint32_t k_mod = MULTI ? K - fdiv(K, a.divH) * H : 0u;

    // row differences of the row just above the run (only used if that row is in the same plane)
    int32_t prev_rd[NSEG][VEC];
#pragma unroll
    for (int s = 0; s < NSEG; ++s)
#pragma unroll
        for (int v = 0; v < VEC; ++v) prev_rd[s][v] = 0;
    if (row_lo > 0) {
        const size_t above = (size_t)(e_lo - W);                  // first element of that row
#pragma unroll
        for (int s = 0; s < NSEG; ++s) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const uint32_t w = (MULTI ? w0 : ((uint32_t)s * kWave + lane) * VEC) + (uint32_t)v;
                const bool on = MULTI ? top_rows : (w < W);
                const float xa = on ? load_elem<IN>(a.x, above + w) : 0.0f;
                const float xl = (on && w > 0) ? load_elem<IN>(a.x, above + w - 1u) : 0.0f;
                const float ta = xa * a.r, tl = xl * a.r;
                const int32_t qa = (fabsf(ta) < 16777216.0f) ? (int32_t)rintf(ta) : 0;
                const int32_t ql = (fabsf(tl) < 16777216.0f) ? (int32_t)rintf(tl) : 0;
                prev_rd[s][v] = (w > 0) ? qa - ql : qa;
            }
        }
    }

    constexpr uint32_t U = NSEG * VEC >= 4 ? 1u : 4u / (NSEG * VEC);   // steps per batch of loads (eight values per lane and batch were slower)
    // FULL batches (every row of the batch inside the run) put the uniform part of the address
    // into the scalar offset of the buffer instruction and know a lane's validity up front;
    // the few steps at the end of a run go through the general form.
    bool col_ok[NSEG];
#pragma unroll
    for (int s = 0; s < NSEG; ++s) col_ok[s] = col[s] != kOob / 4u;
    uint64_t ok_mask[NSEG];
#pragma unroll
    for (int s = 0; s < NSEG; ++s) ok_mask[s] = wave_ballot(col_ok[s]);
    auto fetch = [&](auto full_tag, uint32_t t0, uint32_t t_max, float (&xb)[U][NSEG][VEC]) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t t = (FULL && t0 + u > t_max) ? t_max : t0 + u;   // FULL: never beyond the last full step
            const uint32_t soff = t * stride;                              // uniform
#pragma unroll
            for (int s = 0; s < NSEG; ++s) {
                const int voff = FULL ? (int)(col[s] * ES) : (int)((col[s] + soff) * ES);
                const int sof = FULL ? (int)(soff * ES) : 0;
                if (IN == 0 && VEC == 2) {
                    const u32x2 r = __builtin_amdgcn_raw_buffer_load_b64(r_x, voff, sof, 0);
                    xb[u][s][0] = __uint_as_float(r.x);
                    xb[u][s][VEC - 1] = __uint_as_float(r.y);
                } else if (IN == 0) {
                    xb[u][s][0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r_x, voff, sof, 0));
                } else if (VEC == 2) {
                    const uint32_t r = __builtin_amdgcn_raw_buffer_load_b32(r_x, voff, sof, 0);   // two 16-bit elements
                    xb[u][s][0] = widen16<IN>(r & 0xffffu);
                    xb[u][s][VEC - 1] = widen16<IN>(r >> 16);
                } else {
                    xb[u][s][0] = widen16<IN>((uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r_x, voff, sof, 0));
                }
            }
        }
    };
    uint32_t buffered = 0;                                       // records waiting in s_buf (uniform)
    auto flush_records = [&]() {                                 // s_buf[0 .. buffered) -> rec_dst[cur ...), coalesced
        wave_lds_fence();
        for (uint32_t i = lane; i < buffered; i += kWave) {
            if (cur + i < rec_cap) rec_dst[cur + i] = s_buf[i];
            else if (PASS == 1) atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);
        }
        wave_lds_fence();
        cur += buffered;
        buffered = 0;
    };
    auto flush_oow = [&]() {                                     // the listed codes -> global histogram
        wave_lds_fence();
        // (into the workgroup's partial histogram: the codes just outside the window are few and frequent, and all
        // workgroups adding to one copy of them queue up on a handful of cache lines)
        uint32_t *part = a.hist_parts + (size_t)(blockIdx.x % a.hist_copies) * a.nbins;
        for (uint32_t i = lane; i < cnt.oow_held; i += kWave) atomicAdd(&part[cnt.oow_list[i]], 1u);
        wave_lds_fence();
        cnt.oow_held = 0;
    };
    uint16_t *ring_w = (PASS == 0 && REUSE) ? const_cast<uint16_t *>(enc->ring) : nullptr;
    // REUSE: does the given table have a code word for this code?  From the length table; the single-pass sweep with
    // the whole encode table in LDS reads that instead (an entry is 0 for a symbol without a code word), which saves
    // the length table's LDS.
    auto has_code = [&](uint32_t c) -> bool {
        if (PASS == 0 && REUSE && FULLWIN) return reinterpret_cast<const uint32_t *>(tbl->lds)[2u * c] != 0u;
        return s_len[c] != 0;
    };
    // single-pass compression: encode what the ring holds of the run's first `produced` symbols
    auto drain = [&](uint32_t produced, bool final) {
        if (PASS == 0 && REUSE) {
            if (!final && produced - enc->consumed < 256u) return;
            wave_lds_fence();
            if (a.chunk_syms == 64u) enc->template drain<64, FULLWIN>(*tbl, lane, produced, final);
            else if (a.chunk_syms == 128u) enc->template drain<128, FULLWIN>(*tbl, lane, produced, final);
            else enc->template drain<256, FULLWIN>(*tbl, lane, produced, final);
        }
    };
    auto steps_of = [&](auto full_tag, uint32_t t0, float (&xb)[U][NSEG][VEC]) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t soff = (t0 + u) * stride;
            int32_t carry_q = 0;                                // last column of the previous segment (uniform)
            const uint32_t hmask = h_row ? ~0u : 0u;            // !MULTI: "has a row above"
#pragma unroll
            for (int s = 0; s < NSEG; ++s) {
                const bool valid = FULL ? col_ok[s] : (col[s] + soff < n_el);
                float x[VEC], qf[VEC];
                int32_t q[VEC], rd[VEC], up[VEC], d[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    x[v] = xb[u][s][v];
                    const float t = x[v] * a.r;
                    qf[v] = (fabsf(t) < 16777216.0f) ? rintf(t) : 0.0f;
                    q[v] = (int32_t)qf[v];
                }
                int32_t nql = lane_left(-q[VEC - 1]);           // minus the left neighbour of my first column
                if (MULTI) {
                    rd[0] = first_col ? q[0] : q[0] + nql;
                } else {
                    if (s > 0) nql = (lane == 0u) ? -carry_q : nql;
                    if (NSEG > 1) carry_q = __builtin_amdgcn_readlane(q[VEC - 1], 63);
                    rd[0] = q[0] + nql;
                }
#pragma unroll
                for (int v = 1; v < VEC; ++v) rd[v] = q[v] - q[v - 1];
                if (MULTI) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const int32_t below = __builtin_amdgcn_ds_bpermute((int)((lane - LPR) * 4u), rd[v]);
                        const int32_t upv = top_rows ? prev_rd[0][v] : below;
                        up[v] = h_lane ? upv : 0;
                        prev_rd[0][v] = __builtin_amdgcn_ds_bpermute((int)((lane + (K - 1u) * LPR) * 4u), rd[v]);
                    }
                    h_lane += k_mod;
                    h_lane -= (h_lane >= H) ? H : 0u;
                } else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        up[v] = (int32_t)((uint32_t)prev_rd[s][v] & hmask);
                        prev_rd[s][v] = rd[v];
                    }
                }
                // wavefront masks straight from the comparisons (scalar registers, no per-lane flags)
                const uint64_t vmask = FULL ? ok_mask[s] : wave_ballot(valid);
                uint64_t em[VEC], sm[VEC], any_rec = 0ull;      // lanes with an escape / lanes that failed the fp32 bound filter
                bool inr[VEC], susp[VEC];
                uint32_t code[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    d[v] = (int32_t)((uint32_t)rd[v] - (uint32_t)up[v]);
                    const uint32_t c = (uint32_t)d[v] + (uint32_t)radius;
                    inr[v] = (c - 1u) < code_span;
                    if (REUSE) inr[v] = inr[v] && has_code(inr[v] ? c : 0u);      // no code word in the given table: an escape
                    code[v] = inr[v] ? c : 0u;
                    // error-bound filter: |x - y| in fp32 is within one rounding of the exact error
                    const float err = fabsf(x[v] - qf[v] * a.ebx2);
                    susp[v] = !(err <= eb_lo);                  // also true for NaN / Inf / huge inputs
                    em[v] = wave_ballot(!inr[v]) & vmask;
                    sm[v] = wave_ballot(susp[v]) & vmask;
                    any_rec |= em[v] | sm[v];
                    if (PASS == 0) cnt.nnz_lane += (x[v] != 0.0f) ? 1u : 0u;   // lanes without an element hold 0
                    if (PASS == 0 && !REUSE) {
                        // Histogram: no divergent branch (switching the execution mask costs more than the
                        // atomic).  Lanes that count nothing add to a word of their own; the centre bin is
                        // not counted here, it is what is left of the workgroup's elements.  The window is
                        // replicated: lanes that meet in one bin mostly use different copies.
                        const bool count = valid && code[v] != (uint32_t)radius;
                        if (FULLWIN) {
                            atomicAdd(&s_hist[count ? (code[v] << a.hist_shift) + hist_sub : hist_dummy], 1u);
                        } else {
                            const uint32_t bin = code[v] - a.win_lo;
                            const bool inwin = bin < a.win_n;
                            atomicAdd(&s_hist[(count && inwin) ? (bin << a.hist_shift) + hist_sub : hist_dummy], 1u);
                            // A code outside the window goes to a list in LDS and from there, in bulk, to the global
                            // histogram: an atomic on global memory in this loop would make every step wait for all
                            // loads in flight.
                            const uint64_t om = wave_ballot(count && !inwin);
                            if (om != 0ull) {                   // uniform
                                const uint32_t n_new = (uint32_t)__popcll(om);
                                if (cnt.oow_held + n_new > kQuantOowList) flush_oow();
                                if (count && !inwin)
                                    cnt.oow_list[cnt.oow_held + __builtin_amdgcn_mbcnt_hi((uint32_t)(om >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)om, 0u))] = (uint16_t)code[v];
                                cnt.oow_held += n_new;
                                cnt.oow += n_new;
                            }
                        }
                    }
                }
                if (PASS == 0 && REUSE) {
                    // into the ring (lanes without an element write behind it)
                    const uint32_t at = valid ? ((col[s] + soff) & (kEncRingSyms - 1u)) : kEncRingSyms;
                    if (VEC == 2) *reinterpret_cast<uint32_t *>(ring_w + at) = code[0] | (code[VEC - 1] << 16);
                    else ring_w[at] = (uint16_t)code[0];
                } else if (PASS == 0) {
                    const int voff = FULL ? (int)(col[s] * 2u) : (int)((col[s] + soff) * 2u);
                    const int sof = FULL ? (int)(soff * 2u) : 0;
                    if (VEC == 2) __builtin_amdgcn_raw_buffer_store_b32(code[0] | (code[VEC - 1] << 16), r_c, voff, sof, 0);
                    else __builtin_amdgcn_raw_buffer_store_b16((unsigned short)code[0], r_c, voff, sof, 0);
                }
                // ---- outlier records: escapes and verbatim values, in element order (lanes, then a lane's
                // columns, escape before verbatim).  One wavefront-uniform test per slot.  They go to a small LDS
                // buffer and leave in bulk, so that the loop holds no global store outside this branch. ----
                if (any_rec != 0ull) {
                    if (REUSE && PASS == 0) {                    // an escape, and the table has no code word for it
                        uint64_t any_e = 0ull;
#pragma unroll
                        for (int v = 0; v < VEC; ++v) any_e |= em[v];
                        if (any_e != 0ull && !has_code(0u) && lane == 0) atomicOr(&a.ctl->status, (uint32_t)ST_CODEBOOK);
                    }
                    uint64_t vm[VEC];
                    bool verb[VEC];
                    uint64_t any_s = 0ull;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) { vm[v] = 0ull; verb[v] = false; any_s |= sm[v]; }
                    if (any_s != 0ull) {                         // much rarer than escapes: the exact comparison
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            if (valid && susp[v]) verb[v] = needs_verbatim_rows(x[v], q[v], a.r, a.ebx2, a.eb);
                            vm[v] = wave_ballot(verb[v]);
                        }
                    }
                    uint32_t add = 0, before = 0;                // records of this slot (uniform); those of the lanes below me
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        add += (uint32_t)__popcll(em[v]) + (uint32_t)__popcll(vm[v]);
                        before += __builtin_amdgcn_mbcnt_hi((uint32_t)(em[v] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)em[v], 0u));
                        if (vm[v]) before += __builtin_amdgcn_mbcnt_hi((uint32_t)(vm[v] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)vm[v], 0u));
                        if (PASS == 0) cnt.vrec += (uint32_t)__popcll(vm[v]);
                    }
                    if (add) {
                        if (buffered + add > kQuantRecLds2) flush_records();
                        uint32_t pos = buffered + before;
                        const uint32_t e = e_lo + col[s] + soff;
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            if (valid && !inr[v]) s_buf[pos++] = make_uint2(2u * (e + (uint32_t)v), (uint32_t)d[v]);
                            if (verb[v]) s_buf[pos++] = make_uint2(2u * (e + (uint32_t)v) + 1u, __float_as_uint(x[v]));
                        }
                        buffered += add;
                    }
                }
            }
            if (!MULTI) { ++h_row; h_row = (h_row == H) ? 0u : h_row; }
        }
    };
    // Two batches of steps alternate: the loads of one are in flight while the other is worked on.
    float xa[U][NSEG][VEC], xb[U][NSEG][VEC];
    const std::true_type full{};
    const std::false_type general{};
    const uint32_t n_full = n_steps / (2u * U) * (2u * U);      // steps covered by full double batches
    uint32_t t0 = 0;
    if (n_full) {
        const uint32_t t_max = n_full - 1u;
        fetch(full, 0, t_max, xa);
        for (; t0 < n_full; t0 += 2u * U) {
            fetch(full, t0 + U, t_max, xb);
            steps_of(full, t0, xa);
            drain((t0 + U) * stride, false);
            fetch(full, t0 + 2u * U, t_max, xa);                // the last round re-reads the last step, unused
            steps_of(full, t0 + U, xb);
            drain((t0 + 2u * U) * stride, false);
        }
    }
    for (; t0 < n_steps; t0 += U) {                              // fewer than two batches left
        fetch(general, t0, 0, xa);
        steps_of(general, t0, xa);
        const uint32_t done = (t0 + U) * stride;
        drain(done < n_el ? done : n_el, false);
    }
    drain(n_el, true);
    flush_records();
    if (PASS == 0 && !REUSE && !FULLWIN && cnt.oow_held) flush_oow();
    return cur;
}

// rows [lo, hi) of run `run`
__device__ inline void run_rows(const QuantArgs &a, uint32_t run, uint32_t *lo, uint32_t *hi) {
    const uint64_t r0 = (uint64_t)run * a.rows_per_wave;
    if (r0 >= a.rows_total) { *lo = 0; *hi = 0; return; }
    *lo = (uint32_t)r0;
    *hi = (a.rows_total - *lo < a.rows_per_wave) ? a.rows_total : *lo + a.rows_per_wave;
}

}  // namespace

// One run per wavefront, kQuantBlock / 64 runs per workgroup.
template <int VEC, int NSEG, bool MULTI, bool FULLWIN, bool REUSE, int IN>
__global__ __launch_bounds__(kQuantBlock) void k_quantize_rows(QuantArgs a) {
    extern __shared__ uint32_t s_dyn_qr[];          // histogram window: a.win_n bins, 1 << a.hist_shift copies of each;
                                                    // then one word per thread for the lanes that count nothing
                                                    // (REUSE: the given length table instead, u8[nbins])
    constexpr int kWaves = kQuantBlock / kWave;
    uint32_t *s_hist = s_dyn_qr;
    __shared__ uint64_t s_part64[kWaves];
    __shared__ uint32_t s_tot[kWaves][3];
    __shared__ uint2 s_recbuf[kWaves][kQuantRecLds2];   // outlier records of a wavefront on their way to the staging area

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / kWave));
    uint8_t *s_len = reinterpret_cast<uint8_t *>(s_dyn_qr);
    if (REUSE && (a.ctl->status & (uint32_t)ST_CODEBOOK)) {
        // k_codebook has refused the given table (the same for every thread): nothing is encoded with it, and the
        // kernels behind this one find no records and no words
        if (lane == 0) { a.run_count[blockIdx.x * kWaves + wave] = 0; a.run_words[blockIdx.x * kWaves + wave] = 0; }
        if (tid < 3u) a.run_count[gridDim.x * kWaves + tid * gridDim.x + blockIdx.x] = 0;
        return;
    }
    // REUSE: behind the length table the cached part of the encode table (and a zero entry), then per
    // wavefront the ring of codes (and the word lanes without an element write to) and the assembly buffer
    // (no length table if the whole encode table is there: FULLWIN)
    uint64_t *s_tbl = reinterpret_cast<uint64_t *>(s_len + (FULLWIN ? 0u : ((a.nbins + 7u) & ~7u)));
    uint16_t *s_ring = reinterpret_cast<uint16_t *>(s_tbl + a.enc_n + 1u) + wave * (kEncRingSyms + 4u);
    uint32_t *s_asm = reinterpret_cast<uint32_t *>(reinterpret_cast<uint16_t *>(s_tbl + a.enc_n + 1u) + kWaves * (kEncRingSyms + 4u)) + wave * kEncRunBufWords;
    if (REUSE) {
        if (!FULLWIN)
            for (uint32_t i = tid; i < a.nbins; i += kQuantBlock) s_len[i] = a.reuse_len[i];
        for (uint32_t i = tid; i <= a.enc_n; i += kQuantBlock) s_tbl[i] = (i < a.enc_n) ? a.enc[a.enc_lo + i] : 0ull;
        for (uint32_t i = lane; i < kEncRunBufWords; i += kWave) s_asm[i] = 0;
    } else {
        for (uint32_t i = tid; i < (a.win_n << a.hist_shift); i += kQuantBlock) s_hist[i] = 0;
    }
    __syncthreads();

    const uint32_t run = blockIdx.x * kWaves + wave;
    uint32_t row_lo, row_hi;
    run_rows(a, run, &row_lo, &row_hi);
    SweepCounts cnt;
    // (a window that does not hold every bin: behind it and the threads' dummy words, a list per wavefront)
    if (!REUSE && !FULLWIN) cnt.oow_list = reinterpret_cast<uint16_t *>(s_hist + (a.win_n << a.hist_shift) + kQuantBlock) + wave * kQuantOowList;
    uint32_t my_records = 0;
    RunEncoder enc;
    TableView<FULLWIN> tbl{s_tbl, a.enc, a.enc_lo, a.enc_n, a.nbins};
    if (REUSE) {
        const uint32_t e_lo = row_lo * a.divW.d, n_el = (row_hi - row_lo) * a.divW.d;    // a whole number of chunks, but for the last run
        enc.ring = s_ring; enc.buf = s_asm;
        enc.cap_words = n_el / 2u;
        enc.r_words = rows_rsrc(a.work_words + e_lo / 2u, enc.cap_words * 4u);
        enc.r_chunk = rows_rsrc(a.chunk_off + e_lo / a.chunk_syms, (n_el + a.chunk_syms - 1u) / a.chunk_syms * 4u);
        enc.zero_pair = a.zero_pair;
    }
    if (row_hi > row_lo)
        my_records = sweep_rows<VEC, NSEG, MULTI, FULLWIN, 0, REUSE, IN>(a, row_lo, row_hi, lane, s_hist, (a.win_n << a.hist_shift) + tid, s_recbuf[wave],
                                                                 reinterpret_cast<uint2 *>(a.stage) + (size_t)run * kQuantRecRun, kQuantRecRun, cnt, s_len,
                                                                 REUSE ? &enc : nullptr, REUSE ? &tbl : nullptr);
    if (REUSE) {
        if (lane == 0) a.run_words[run] = enc.wrun;
        // a run that needs more than 16 bits per symbol does not fit its work area: the table does not suit this tensor
        if (wave_ballot(enc.overflow) && lane == 0) atomicOr(&a.ctl->status, (uint32_t)ST_CODEBOOK);
    }
    // results: record count per run; records, non-zero inputs and verbatim records per workgroup (summed
    // up by the gather kernel; thousands of atomics on one counter would cost more than the sweep)
    const uint32_t nnz_wave = wave_sum<uint32_t>(cnt.nnz_lane);
    if (lane == 0) {
        a.run_count[run] = my_records;
        s_tot[wave][0] = my_records; s_tot[wave][1] = nnz_wave; s_tot[wave][2] = cnt.vrec;
    }

    // ---- flush the private histogram ----
    // Into one of several partial histograms: the occupied bins are a few cache lines, and thousands
    // of workgroups adding to the same lines would queue up behind each other for longer than the
    // sweep takes.  k_gather_records adds the copies up.
    // centre bin = elements of the workgroup - everything counted elsewhere
    __syncthreads();
    if (tid < 3u) {
        uint32_t t = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) t += s_tot[w][tid];
        a.run_count[gridDim.x * kWaves + tid * gridDim.x + blockIdx.x] = t;   // three arrays of one entry per workgroup
    }
    if (REUSE) return;                              // no histogram (uniform: every thread has passed the barrier above)
    uint32_t *part = a.hist_parts + (size_t)(blockIdx.x % a.hist_copies) * a.nbins;
    uint64_t counted = (FULLWIN || lane != 0u) ? 0ull : (uint64_t)cnt.oow;
    for (uint32_t i = tid; i < a.win_n; i += kQuantBlock) {
        uint32_t v = 0;
        for (uint32_t k = 0; k < (1u << a.hist_shift); ++k) v += s_hist[(i << a.hist_shift) + k];
        counted += v;
        if (v) atomicAdd(&part[a.win_lo + i], v);
    }
    uint64_t total;
    (void)block_excl_scan<uint64_t, kWaves>(counted, s_part64, total);
    if (tid == 0) {
        const uint64_t r0 = (uint64_t)blockIdx.x * kWaves * a.rows_per_wave;
        uint64_t r1 = r0 + (uint64_t)kWaves * a.rows_per_wave;
        if (r1 > a.rows_total) r1 = a.rows_total;
        const uint64_t elems = (r1 > r0) ? (r1 - r0) * a.divW.d : 0ull;
        if (elems > total) atomicAdd(&part[a.radius], (uint32_t)(elems - total));
    }
}

// Moves the staged records of every run to their final, ordered place; same grid as k_quantize_rows.
template <int VEC, int NSEG, bool MULTI, bool REUSE, int IN>
__global__ __launch_bounds__(kQuantBlock) void k_gather_records(QuantArgs a) {
    constexpr int kWaves = kQuantBlock / kWave;
    extern __shared__ uint32_t s_dyn_gr[];          // REUSE: the given length table, u8[nbins] (for runs that are swept again)
    __shared__ uint64_t s_part64[kWaves];
    __shared__ uint2 s_recbuf[kWaves][kQuantRecLds2];
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = (uint32_t)lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / kWave));
    const uint32_t n_runs = gridDim.x * kWaves;
    const uint32_t run0 = blockIdx.x * kWaves;

    uint8_t *s_len = reinterpret_cast<uint8_t *>(s_dyn_gr);
    if (REUSE) {
        for (uint32_t i = tid; i < a.nbins; i += kQuantBlock) s_len[i] = a.reuse_len[i];
        __syncthreads();
    }
    // histogram: one thread per bin adds up the partial histograms (codes outside the LDS window of
    // the quantise kernel were counted in hist directly)
    for (uint32_t b = blockIdx.x * kQuantBlock + tid; !REUSE && b < a.nbins; b += gridDim.x * kQuantBlock) {
        uint32_t v = a.hist[b];                                             // (codes outside the LDS window)
        uint32_t p[kQuantHistCopiesMax];                                    // every copy in flight at once: one round trip
#pragma unroll
        for (uint32_t j = 0; j < kQuantHistCopiesMax; ++j) p[j] = (j < a.hist_copies) ? a.hist_parts[(size_t)j * a.nbins + b] : 0u;
#pragma unroll
        for (uint32_t j = 0; j < kQuantHistCopiesMax; ++j) v += p[j];
        a.hist[b] = v;
    }

    // sum of the per-workgroup counters wg[0 .. count) over the workgroup, eight loads in flight per thread
    auto total_of = [&](const uint32_t *wg, uint32_t count) {
        uint64_t sum = 0;
        for (uint32_t i0 = 0; i0 < count; i0 += 8u * kQuantBlock) {
            uint32_t v[8];
#pragma unroll
            for (uint32_t j = 0; j < 8; ++j) {
                const uint32_t i = i0 + j * kQuantBlock + tid;
                v[j] = (i < count) ? wg[i] : 0u;
            }
#pragma unroll
            for (uint32_t j = 0; j < 8; ++j) sum += v[j];
        }
        uint64_t total;
        (void)block_excl_scan<uint64_t, kWaves>(sum, s_part64, total);
        return total;
    };
    const uint32_t *wg_rec = a.run_count + n_runs, *wg_nnz = wg_rec + gridDim.x, *wg_vrec = wg_nnz + gridDim.x;
    // records of all workgroups in front of mine
    uint64_t base = total_of(wg_rec, blockIdx.x);
    uint32_t mine = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t c = a.run_count[run0 + w];
        if ((uint32_t)w < wave) base += c;
        if ((uint32_t)w == wave) mine = c;
    }
    if (blockIdx.x + 1u == gridDim.x && tid == kQuantBlock - 1) a.ctl->n_rec = base + mine;   // last run: base covers all runs before it
    // two of the first workgroups (little in front of them) total the other counters, one each
    if (blockIdx.x == 0) {
        const uint64_t nnz_total = total_of(wg_nnz, gridDim.x);
        if (tid == 0) a.ctl->nnz = nnz_total;
    }
    if (blockIdx.x == (gridDim.x > 1u ? 1u : 0u)) {
        const uint64_t vrec_total = total_of(wg_vrec, gridDim.x);
        if (tid == 0) a.ctl->n_vrec = vrec_total;
    }
    if (!mine) return;
    const uint32_t run = run0 + wave;
    uint2 *dst = reinterpret_cast<uint2 *>(a.rec) + base;
    const uint64_t room = (base < a.rec_cap) ? a.rec_cap - base : 0ull;
    if (mine <= kQuantRecRun) {
        const uint2 *src = reinterpret_cast<const uint2 *>(a.stage) + (size_t)run * kQuantRecRun;
        for (uint32_t i = lane; i < mine; i += kWave) {
            if (i < room) dst[i] = src[i];
            else atomicOr(&a.ctl->status, (uint32_t)ST_CAPACITY);
        }
    } else {
        // more outliers than the staging area of a run holds: derive them again, in place
        uint32_t row_lo, row_hi;
        run_rows(a, run, &row_lo, &row_hi);
        SweepCounts unused;
        (void)sweep_rows<VEC, NSEG, MULTI, true, 1, REUSE, IN>(a, row_lo, row_hi, lane, nullptr, 0, s_recbuf[wave], dst, room, unused, s_len);
    }
}

#define COMET_INST_QR(VEC, NSEG, MULTI)                                                          \
    template __global__ void k_quantize_rows<VEC, NSEG, MULTI, true, false, 0>(QuantArgs);       \
    template __global__ void k_quantize_rows<VEC, NSEG, MULTI, false, false, 0>(QuantArgs);      \
    template __global__ void k_quantize_rows<VEC, NSEG, MULTI, true, true, 0>(QuantArgs);        \
    template __global__ void k_quantize_rows<VEC, NSEG, MULTI, false, true, 0>(QuantArgs);       \
    template __global__ void k_gather_records<VEC, NSEG, MULTI, false, 0>(QuantArgs);            \
    template __global__ void k_gather_records<VEC, NSEG, MULTI, true, 0>(QuantArgs);             \
    COMET_INST_QR16(VEC, NSEG, MULTI, 1)                                                         \
    COMET_INST_QR16(VEC, NSEG, MULTI, 2)
#define COMET_INST_QR16(VEC, NSEG, MULTI, IN)                                                    \
    template __global__ void k_quantize_rows<VEC, NSEG, MULTI, true, false, IN>(QuantArgs);      \
    template __global__ void k_quantize_rows<VEC, NSEG, MULTI, false, false, IN>(QuantArgs);     \
    template __global__ void k_gather_records<VEC, NSEG, MULTI, false, IN>(QuantArgs);
COMET_INST_QR(1, 1, true)
COMET_INST_QR(1, 1, false)
COMET_INST_QR(1, 2, false)
COMET_INST_QR(1, 4, false)
COMET_INST_QR(1, 8, false)
COMET_INST_QR(2, 1, true)
COMET_INST_QR(2, 1, false)
COMET_INST_QR(2, 2, false)
COMET_INST_QR(2, 4, false)
#undef COMET_INST_QR16
#undef COMET_INST_QR

}  // namespace comet
