/*
 * comet_oracle.c -- plain, slow, single-threaded CPU reference of the COMET
 * activation codec (error-bounded SZ-style compressor / decompressor).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the HIP library can be checked
 * bit for bit.  Only the tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it; the product path never does.  It shares no code, header,
 * table or constant generator with the HIP sources.
 *
 * What the paper fixes (COMET, Sec. 2.2, Sec. 3.4, Sec. 4.1):
 *   - stage order: quantise the fp32 input against the error bound
 *     ("dual-quantisation"), predict every point from its neighbours with a
 *     Lorenzo predictor, emit one integer quantisation code per value, Huffman
 *     code all quantisation codes (Sec. 4.1);
 *   - the error-bounded mode: |x - xhat| never exceeds the absolute bound eb
 *     (Sec. 2.2);
 *   - the re-zero filter added to decompression: every reconstructed value whose
 *     distance to zero is within eb is returned as exactly zero (Sec. 3.4);
 *   - the adaptive bound: sigma = 0.01 * M_average (Sec. 3.2) and
 *     eb = sigma / (a * Lbar * sqrt(N * R)) (Sec. 3.3), a = 0.32 (Sec. 5.2).
 * Everything the paper leaves open (rounding mode, bin count, tie rule of the
 * Huffman tree, chunking, bit order, container layout) follows the readings
 * listed in the design notes of this repository; each is restated where it is
 * implemented below.
 *
 * Pins (tests/test_oracle_*.py): two hand-computed pipelines, numpy rint /
 * cumsum / bincount identities, an independent heap Huffman cost, Kraft sums,
 * closed-form code lengths, the error-bound invariant, brute-force tie cases,
 * a hand-computed container with an elided chunk.
 * Parity unpinned: anything about real network activations (the paper's
 * Table 1 ratios) -- the datasets are not available.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_ERR_INVALID (-1)
#define ORC_ERR_CAPACITY (-2)
#define ORC_ERR_FORMAT (-3)
#define ORC_ERR_NOMEM (-5)

#define ORC_MAGIC 0x31544D43u /* bytes 'C','M','T','1' */
#define ORC_HEADER_BYTES 128u

/* ------------------------------------------------------------------------- */
/* argument checks shared by the whole-pipeline entry points                  */
/* ------------------------------------------------------------------------- */

static int valid_eb(float eb) {
    /* finite and inside [2^-100, 2^100] so that 2*eb and 1/(2*eb) are normal */
    return isfinite(eb) && eb >= 0x1p-100f && eb <= 0x1p100f;
}

static int valid_nbins(uint32_t nbins) {
    return nbins >= 4u && nbins <= 65536u && (nbins % 2u) == 0u;
}

/* n = N*C*H*W must be in [1, 2^31): the outlier list spends one key bit on the
 * record type. */
static int shape_elems(uint32_t N, uint32_t C, uint32_t H, uint32_t W, uint64_t *n) {
    if (!N || !C || !H || !W) return 0;
    uint64_t a = (uint64_t)N * C;
    uint64_t b = (uint64_t)H * W;
    if (a >= (1ull << 31) || b >= (1ull << 31)) return 0;
    uint64_t t = a * b;
    if (t >= (1ull << 31)) return 0;
    *n = t;
    return 1;
}

static uint32_t f2u(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float u2f(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* Constants derived from eb once, on the host, in this order (Sec. 4.1 leaves
 * the arithmetic open; reading: multiply by a precomputed reciprocal). */
void oracle_constants(float eb, float *ebx2, float *r) {
    *ebx2 = 2.0f * eb;                       /* exact: a power-of-two scaling */
    *r = (float)(1.0 / (double)(*ebx2));     /* fp64 divide, one rounding to fp32 */
}

/* ------------------------------------------------------------------------- */
/* Step 1: prequantisation ("dual-quantisation", first half; Sec. 4.1)        */
/* ------------------------------------------------------------------------- */
/*
 * t = x * r in fp32, q = round-half-to-even(t).  The bound of Sec. 2.2 is then
 * verified per element in fp64 on the value the decompressor will produce,
 * fl32(q * 2eb); an element that fails, or whose t is not a finite number below
 * 2^24 in magnitude, is flagged as a value-outlier (stored verbatim later).
 * Non-representable t gives q = 0; a failing finite element keeps its q so its
 * neighbours still predict from it.
 */
static int prequant_impl(const float *x, uint64_t n, float eb, int zero_first,
                         int32_t *q, uint8_t *is_value_outlier, uint64_t *nnz) {
    if (!x || !q || !is_value_outlier || !valid_eb(eb)) return ORC_ERR_INVALID;
    float ebx2, r;
    oracle_constants(eb, &ebx2, &r);
    uint64_t nz = 0;
    for (uint64_t i = 0; i < n; ++i) {
        float xi = x[i];
        if (xi != 0.0f) ++nz;               /* NaN counts as non-zero */
        if (zero_first && fabsf(xi) <= eb) { /* the alternative of Sec. 3.4 (see below); NaN fails the comparison */
            q[i] = 0;
            is_value_outlier[i] = 0;
            continue;
        }
        float t = xi * r;
        if (!(fabsf(t) < 16777216.0f)) {    /* also true for NaN and Inf */
            q[i] = 0;
            is_value_outlier[i] = 1;
            continue;
        }
        int32_t qi = (int32_t)rintf(t);     /* default rounding mode: ties to even */
        float y = (float)qi * ebx2;
        double err = fabs((double)xi - (double)y);
        q[i] = qi;
        is_value_outlier[i] = (err <= (double)eb) ? 0 : 1;
    }
    if (nnz) *nnz = nz;
    return ORC_OK;
}

int oracle_prequant(const float *x, uint64_t n, float eb,
                    int32_t *q, uint8_t *is_value_outlier, uint64_t *nnz) {
    return prequant_impl(x, n, eb, 0, q, is_value_outlier, nnz);
}

/*
 * The alternative zero handling that Sec. 3.4 describes and turns down: every
 * value within eb of zero is set to zero already in the first quantisation
 * step, instead of being filtered after reconstruction.  With prequantisation
 * on the lattice of multiples of 2eb this is the same thing: r is within half
 * an ulp of 1/(2eb), so eb * r rounds to at most 1/2 (a tie goes to the even
 * neighbour, 1/2 itself), multiplication is monotonic, and |x * r| <= 1/2
 * rounds to q = 0, which is within the bound of x.  The switch therefore
 * changes no quantised value; it exists so that this can be checked.
 */
int oracle_prequant_zero_first(const float *x, uint64_t n, float eb,
                               int32_t *q, uint8_t *is_value_outlier, uint64_t *nnz) {
    return prequant_impl(x, n, eb, 1, q, is_value_outlier, nnz);
}

/* ------------------------------------------------------------------------- */
/* Step 2: 2-D Lorenzo prediction and quantisation codes (Sec. 4.1)           */
/* ------------------------------------------------------------------------- */
/*
 * Per (n,c) plane of H x W, with q = 0 outside the plane:
 *   d(h,w) = q(h,w) - q(h,w-1) - q(h-1,w) + q(h-1,w-1)
 * in wrap-around 32-bit arithmetic.  radius = nbins/2.  If -radius < d < radius
 * the code is d + radius (1 .. nbins-1); otherwise the code is 0, the escape
 * symbol, and d itself goes to the outlier list.  delta[] receives every d.
 */
int oracle_predict_code(const int32_t *q, uint32_t N, uint32_t C, uint32_t H, uint32_t W,
                        uint32_t nbins, uint16_t *codes, int32_t *delta) {
    uint64_t n;
    if (!q || !codes || !valid_nbins(nbins) || !shape_elems(N, C, H, W, &n)) return ORC_ERR_INVALID;
    const int32_t radius = (int32_t)(nbins / 2u);
    const uint64_t planes = (uint64_t)N * C;
    for (uint64_t p = 0; p < planes; ++p) {
        const int32_t *qp = q + p * (uint64_t)H * W;
        for (uint32_t h = 0; h < H; ++h) {
            for (uint32_t w = 0; w < W; ++w) {
                uint32_t here = (uint32_t)qp[(uint64_t)h * W + w];
                uint32_t left = (w > 0) ? (uint32_t)qp[(uint64_t)h * W + (w - 1)] : 0u;
                uint32_t up = (h > 0) ? (uint32_t)qp[(uint64_t)(h - 1) * W + w] : 0u;
                uint32_t upleft = (h > 0 && w > 0) ? (uint32_t)qp[(uint64_t)(h - 1) * W + (w - 1)] : 0u;
                int32_t d = (int32_t)(here - left - up + upleft);
                uint64_t i = p * (uint64_t)H * W + (uint64_t)h * W + w;
                if (delta) delta[i] = d;
                if (d > -radius && d < radius) codes[i] = (uint16_t)(d + radius);
                else codes[i] = 0;
            }
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Step 3: histogram of the quantisation codes                                */
/* ------------------------------------------------------------------------- */
int oracle_histogram(const uint16_t *codes, uint64_t n, uint32_t nbins, uint32_t *freq) {
    if (!codes || !freq || !valid_nbins(nbins)) return ORC_ERR_INVALID;
    memset(freq, 0, (size_t)nbins * sizeof(uint32_t));
    for (uint64_t i = 0; i < n; ++i) {
        if (codes[i] >= nbins) return ORC_ERR_INVALID;
        freq[codes[i]] += 1u;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Step 4: Huffman code lengths (Sec. 4.1 "customized Huffman coding")        */
/* ------------------------------------------------------------------------- */
/*
 * Textbook two-queue construction on the symbols with freq > 0:
 *   - leaves sorted ascending by (freq, symbol);
 *   - internal nodes are appended to a FIFO in creation order;
 *   - each of the m-1 steps removes the two smallest heads, preferring the leaf
 *     when a leaf and an internal node weigh the same, and appends their sum;
 *   - the length of a symbol is the depth of its leaf.
 * One active symbol gets length 1.  Symbols with freq 0 get length 0.
 * Reading for the longest code (the paper gives none): 57 bits, the longest code
 * word that shares a 64-bit table entry with its 6-bit length; a histogram whose
 * tree is deeper is refused.  A leaf at depth d needs a total count of at least
 * Fibonacci(d + 2), and Fibonacci(60) > 2^40, so no tensor of fewer than 2^31
 * elements gets there; only a hand-made histogram can.
 */
typedef struct { uint64_t f; uint32_t s; } orc_leaf;

static int leaf_cmp(const void *a, const void *b) {
    const orc_leaf *x = (const orc_leaf *)a, *y = (const orc_leaf *)b;
    if (x->f != y->f) return (x->f < y->f) ? -1 : 1;
    if (x->s != y->s) return (x->s < y->s) ? -1 : 1;
    return 0;
}

int oracle_code_lengths(const uint32_t *freq, uint32_t nbins, uint8_t *len) {
    if (!freq || !len || nbins == 0 || nbins > 65536u) return ORC_ERR_INVALID;
    memset(len, 0, nbins);
    uint32_t m = 0;
    for (uint32_t s = 0; s < nbins; ++s) if (freq[s]) ++m;
    if (m == 0) return ORC_OK;
    orc_leaf *leaf = (orc_leaf *)malloc((size_t)m * sizeof(orc_leaf));
    uint64_t *iw = (uint64_t *)malloc((size_t)m * sizeof(uint64_t));   /* internal weights */
    uint32_t *leaf_parent = (uint32_t *)malloc((size_t)m * sizeof(uint32_t));
    uint32_t *int_parent = (uint32_t *)malloc((size_t)m * sizeof(uint32_t));
    uint32_t *int_depth = (uint32_t *)malloc((size_t)m * sizeof(uint32_t));
    if (!leaf || !iw || !leaf_parent || !int_parent || !int_depth) {
        free(leaf); free(iw); free(leaf_parent); free(int_parent); free(int_depth);
        return ORC_ERR_NOMEM;
    }
    uint32_t k = 0;
    for (uint32_t s = 0; s < nbins; ++s) if (freq[s]) { leaf[k].f = freq[s]; leaf[k].s = s; ++k; }
    qsort(leaf, m, sizeof(orc_leaf), leaf_cmp);
    int rc = ORC_OK;
    if (m == 1) {
        len[leaf[0].s] = 1;
    } else {
        uint32_t li = 0;      /* head of the leaf queue */
        uint32_t ii = 0;      /* head of the internal-node queue */
        uint32_t ni = 0;      /* internal nodes created so far */
        for (uint32_t step = 0; step + 1 < m; ++step) {
            uint64_t sum = 0;
            for (int pick = 0; pick < 2; ++pick) {
                int take_leaf;
                if (li < m && ii < ni) take_leaf = (leaf[li].f <= iw[ii]);   /* tie: leaf first */
                else take_leaf = (li < m);
                if (take_leaf) { sum += leaf[li].f; leaf_parent[li] = ni; ++li; }
                else { sum += iw[ii]; int_parent[ii] = ni; ++ii; }
            }
            iw[ni++] = sum;
        }
        /* ni == m-1; the last internal node is the root */
        int_depth[ni - 1] = 0;
        for (uint32_t j = ni - 1; j-- > 0;) int_depth[j] = int_depth[int_parent[j]] + 1u;
        for (uint32_t i = 0; i < m; ++i) {
            uint32_t dpt = int_depth[leaf_parent[i]] + 1u;
            if (dpt > 57u) { rc = ORC_ERR_INVALID; break; }
            len[leaf[i].s] = (uint8_t)dpt;
        }
    }
    free(leaf); free(iw); free(leaf_parent); free(int_parent); free(int_depth);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Step 5: canonical codes                                                    */
/* ------------------------------------------------------------------------- */
/*
 * Active symbols ordered ascending by (length, symbol).  The first gets code 0
 * of its length; each next one gets (previous + 1) << (its length - previous
 * length).  A code is the low `len` bits of code[s], read from the most
 * significant of those bits first.
 */
int oracle_canonical_codes(const uint8_t *len, uint32_t nbins, uint64_t *code) {
    if (!len || !code || nbins == 0 || nbins > 65536u) return ORC_ERR_INVALID;
    memset(code, 0, (size_t)nbins * sizeof(uint64_t));
    uint64_t prev_code = 0;
    uint32_t prev_len = 0;
    int first = 1;
    for (uint32_t L = 1; L <= 64u; ++L) {
        for (uint32_t s = 0; s < nbins; ++s) {
            if (len[s] != L) continue;
            if (first) { prev_code = 0; first = 0; }
            else {
                prev_code = prev_code + 1u;
                uint32_t sh = L - prev_len;
                prev_code = (sh >= 64u) ? 0 : (prev_code << sh);
            }
            prev_len = L;
            code[s] = prev_code;
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Step 6: chunked encode                                                     */
/* ------------------------------------------------------------------------- */
/*
 * Symbols in linear index order are cut into chunks of chunk_syms (the last one
 * may be shorter).  A chunk's bit string is the concatenation of its codes, each
 * most-significant bit first.  Stream bit k of a chunk sits at bit 31 - (k % 32)
 * of its word k / 32; the last word of a chunk is padded with zero bits.  Chunk
 * j starts at word chunk_off[j] = sum over i<j of ceil(bits_i / 32).
 */
static void put_bit(uint32_t *words, uint64_t bitpos, uint32_t bit) {
    if (bit) words[bitpos / 32u] |= (1u << (31u - (uint32_t)(bitpos % 32u)));
}

/*
 * zero_chunks (container version 2): a chunk all of whose codes are the centre
 * code nbins/2 -- residual zero everywhere, which is what a region of zeros
 * (or of any constant) gives after prediction -- takes no words at all.  The
 * sparsity of activations behind ReLU (Sec. 4.2, the ratio R) makes such
 * chunks common.  A chunk with symbols in it otherwise has at least one bit, so a
 * word count of zero is unambiguous and the chunk table needs no flag.  The
 * histogram and the code lengths are those of all codes, elided or not.
 */
static int encode_impl(const uint16_t *codes, uint64_t n, uint32_t nbins, uint32_t chunk_syms,
                  const uint8_t *len, const uint64_t *code, int zero_chunks,
                  uint32_t *chunk_off, uint64_t n_chunks_cap,
                  uint32_t *payload, uint64_t payload_cap_words, uint64_t *payload_words) {
    if (!codes || !len || !code || !chunk_off || !payload_words || chunk_syms == 0) return ORC_ERR_INVALID;
    uint64_t n_chunks = (n + chunk_syms - 1u) / chunk_syms;
    if (n_chunks > n_chunks_cap) return ORC_ERR_CAPACITY;
    uint64_t word = 0;
    for (uint64_t j = 0; j < n_chunks; ++j) {
        uint64_t lo = j * chunk_syms;
        uint64_t hi = lo + chunk_syms; if (hi > n) hi = n;
        uint64_t bits = 0;
        for (uint64_t i = lo; i < hi; ++i) {
            if (codes[i] >= nbins || len[codes[i]] == 0) return ORC_ERR_INVALID;
            bits += len[codes[i]];
        }
        if (zero_chunks) {
            int all_centre = 1;
            for (uint64_t i = lo; i < hi; ++i) if (codes[i] != nbins / 2u) all_centre = 0;
            if (all_centre) bits = 0;
        }
        uint64_t words = (bits + 31u) / 32u;
        if (word > 0xFFFFFFFFull) return ORC_ERR_CAPACITY;
        chunk_off[j] = (uint32_t)word;
        if (word + words > payload_cap_words) return ORC_ERR_CAPACITY;
        if (payload && words) {
            for (uint64_t k = 0; k < words; ++k) payload[word + k] = 0u;
            uint64_t bp = 0;
            for (uint64_t i = lo; i < hi; ++i) {
                uint32_t L = len[codes[i]];
                uint64_t cw = code[codes[i]];
                for (uint32_t b = 0; b < L; ++b) {
                    uint32_t bit = (uint32_t)((cw >> (L - 1u - b)) & 1u);
                    put_bit(payload + word, bp++, bit);
                }
            }
        }
        word += words;
    }
    *payload_words = word;
    return ORC_OK;
}

int oracle_encode(const uint16_t *codes, uint64_t n, uint32_t nbins, uint32_t chunk_syms,
                  const uint8_t *len, const uint64_t *code,
                  uint32_t *chunk_off, uint64_t n_chunks_cap,
                  uint32_t *payload, uint64_t payload_cap_words, uint64_t *payload_words) {
    return encode_impl(codes, n, nbins, chunk_syms, len, code, 0, chunk_off, n_chunks_cap, payload, payload_cap_words, payload_words);
}

int oracle_encode_zero_chunks(const uint16_t *codes, uint64_t n, uint32_t nbins, uint32_t chunk_syms,
                              const uint8_t *len, const uint64_t *code,
                              uint32_t *chunk_off, uint64_t n_chunks_cap,
                              uint32_t *payload, uint64_t payload_cap_words, uint64_t *payload_words) {
    return encode_impl(codes, n, nbins, chunk_syms, len, code, 1, chunk_off, n_chunks_cap, payload, payload_cap_words, payload_words);
}

/* ------------------------------------------------------------------------- */
/* Step 7: chunk decode                                                       */
/* ------------------------------------------------------------------------- */
/*
 * Canonical decoding straight from the lengths: for every length L keep the
 * first code of that length and how many symbols have it; read bits one at a
 * time, extending the candidate code, until it falls inside the range of its
 * length.  Each chunk must consume exactly its words, and its padding bits
 * must be zero.  zero_chunks (container version 2): a chunk without words is
 * the centre code nbins/2 throughout.
 */
static int decode_impl(const uint8_t *len, uint32_t nbins, int zero_chunks,
                  const uint32_t *chunk_off, const uint32_t *payload, uint64_t payload_words,
                  uint64_t n, uint32_t chunk_syms, uint16_t *codes_out) {
    if (!len || !chunk_off || !codes_out || chunk_syms == 0 || nbins == 0 || nbins > 65536u) return ORC_ERR_INVALID;
    uint64_t count[65]; uint64_t first_code[65]; uint64_t first_index[65];
    memset(count, 0, sizeof(count));
    uint32_t n_active = 0;
    for (uint32_t s = 0; s < nbins; ++s) {
        if (len[s] > 64u) return ORC_ERR_FORMAT;
        if (len[s]) { count[len[s]]++; ++n_active; }
    }
    if (n_active == 0) return (n == 0) ? ORC_OK : ORC_ERR_FORMAT;
    uint32_t *sorted = (uint32_t *)malloc((size_t)n_active * sizeof(uint32_t));
    if (!sorted) return ORC_ERR_NOMEM;
    {
        uint32_t k = 0;
        for (uint32_t L = 1; L <= 64u; ++L)
            for (uint32_t s = 0; s < nbins; ++s) if (len[s] == L) sorted[k++] = s;
    }
    {
        /* first code of each length by the canonical recurrence */
        uint64_t c = 0; uint64_t idx = 0; int started = 0; uint32_t prevL = 0;
        for (uint32_t L = 1; L <= 64u; ++L) {
            first_code[L] = 0; first_index[L] = idx;
            if (!count[L]) continue;
            if (!started) { c = 0; started = 1; }
            else { uint32_t sh = L - prevL; c = (sh >= 64u) ? 0 : (c << sh); }
            first_code[L] = c;
            c += count[L];        /* one past the last code of this length */
            idx += count[L];
            prevL = L;
        }
    }
    uint64_t n_chunks = (n + chunk_syms - 1u) / chunk_syms;
    int rc = ORC_OK;
    for (uint64_t j = 0; j < n_chunks && rc == ORC_OK; ++j) {
        uint64_t lo = j * chunk_syms;
        uint64_t hi = lo + chunk_syms; if (hi > n) hi = n;
        uint64_t w0 = chunk_off[j];
        uint64_t w1 = (j + 1 < n_chunks) ? chunk_off[j + 1] : payload_words;
        if (w0 > w1 || w1 > payload_words) { rc = ORC_ERR_FORMAT; break; }
        if (zero_chunks && w0 == w1) {
            for (uint64_t i = lo; i < hi; ++i) codes_out[i] = (uint16_t)(nbins / 2u);
            continue;
        }
        uint64_t nbits_avail = (w1 - w0) * 32u;
        uint64_t bp = 0;
        for (uint64_t i = lo; i < hi; ++i) {
            uint64_t c = 0; uint32_t L = 0; int found = 0;
            while (L < 64u) {
                if (bp >= nbits_avail) break;
                uint32_t bit = (payload[w0 + bp / 32u] >> (31u - (uint32_t)(bp % 32u))) & 1u;
                ++bp; ++L;
                c = (c << 1) | bit;
                if (count[L] && c >= first_code[L] && c - first_code[L] < count[L]) {
                    codes_out[i] = (uint16_t)sorted[first_index[L] + (c - first_code[L])];
                    found = 1;
                    break;
                }
            }
            if (!found) { rc = ORC_ERR_FORMAT; break; }
        }
        if (rc != ORC_OK) break;
        if ((bp + 31u) / 32u != (w1 - w0)) { rc = ORC_ERR_FORMAT; break; }
        for (; bp < nbits_avail; ++bp)
            if ((payload[w0 + bp / 32u] >> (31u - (uint32_t)(bp % 32u))) & 1u) { rc = ORC_ERR_FORMAT; break; }
    }
    free(sorted);
    return rc;
}

int oracle_decode(const uint8_t *len, uint32_t nbins,
                  const uint32_t *chunk_off, const uint32_t *payload, uint64_t payload_words,
                  uint64_t n, uint32_t chunk_syms, uint16_t *codes_out) {
    return decode_impl(len, nbins, 0, chunk_off, payload, payload_words, n, chunk_syms, codes_out);
}

int oracle_decode_zero_chunks(const uint8_t *len, uint32_t nbins,
                              const uint32_t *chunk_off, const uint32_t *payload, uint64_t payload_words,
                              uint64_t n, uint32_t chunk_syms, uint16_t *codes_out) {
    return decode_impl(len, nbins, 1, chunk_off, payload, payload_words, n, chunk_syms, codes_out);
}

/* ------------------------------------------------------------------------- */
/* Step 8: Lorenzo reconstruction, dequantisation, re-zero filter             */
/* ------------------------------------------------------------------------- */
/*
 * d = code - radius, or the listed value where code == 0 (escape).  Per plane,
 * q(h,w) = sum of d(i,j) over i <= h, j <= w, in wrap-around int32.
 * xhat = fl32(q) * 2eb in fp32; value-outlier records overwrite xhat with their
 * stored bit pattern; last, the filter of Sec. 3.4: |xhat| <= eb gives +0.0f
 * (NaN fails the comparison and is kept).
 *
 * Outlier records: (key, payload) pairs sorted by key; key = 2*index + type;
 * type 0 carries d (int32), type 1 carries the fp32 bit pattern.
 */
int oracle_reconstruct(const uint16_t *codes, const uint32_t *rec, uint64_t n_rec,
                       uint32_t N, uint32_t C, uint32_t H, uint32_t W, uint32_t nbins,
                       float eb, float *xhat) {
    uint64_t n;
    if (!codes || !xhat || !valid_nbins(nbins) || !valid_eb(eb) || !shape_elems(N, C, H, W, &n)) return ORC_ERR_INVALID;
    if (n_rec && !rec) return ORC_ERR_INVALID;
    float ebx2, r;
    oracle_constants(eb, &ebx2, &r);
    const int32_t radius = (int32_t)(nbins / 2u);
    int32_t *d = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    if (!d) return ORC_ERR_NOMEM;
    for (uint64_t i = 0; i < n; ++i) {
        if (codes[i] >= nbins) { free(d); return ORC_ERR_FORMAT; }
        d[i] = (int32_t)codes[i] - radius;   /* escape placeholders are overwritten below */
    }
    /* every escape must have exactly one type-0 record and vice versa */
    uint64_t n_escape = 0, n_type0 = 0;
    for (uint64_t i = 0; i < n; ++i) if (codes[i] == 0) ++n_escape;
    uint64_t prev_key = 0;
    for (uint64_t k = 0; k < n_rec; ++k) {
        uint32_t key = rec[2 * k];
        uint64_t idx = key >> 1;
        if (k > 0 && key <= prev_key) { free(d); return ORC_ERR_FORMAT; }
        prev_key = key;
        if (idx >= n) { free(d); return ORC_ERR_FORMAT; }
        if ((key & 1u) == 0u) {
            if (codes[idx] != 0) { free(d); return ORC_ERR_FORMAT; }
            d[idx] = (int32_t)rec[2 * k + 1];
            ++n_type0;
        }
    }
    if (n_type0 != n_escape) { free(d); return ORC_ERR_FORMAT; }
    const uint64_t planes = (uint64_t)N * C;
    for (uint64_t p = 0; p < planes; ++p) {
        int32_t *dp = d + p * (uint64_t)H * W;
        float *xp = xhat + p * (uint64_t)H * W;
        /* inclusive prefix sums along W, then along H, in place (d becomes q) */
        for (uint32_t h = 0; h < H; ++h)
            for (uint32_t w = 1; w < W; ++w)
                dp[(uint64_t)h * W + w] = (int32_t)((uint32_t)dp[(uint64_t)h * W + w] + (uint32_t)dp[(uint64_t)h * W + w - 1]);
        for (uint32_t h = 1; h < H; ++h)
            for (uint32_t w = 0; w < W; ++w)
                dp[(uint64_t)h * W + w] = (int32_t)((uint32_t)dp[(uint64_t)h * W + w] + (uint32_t)dp[(uint64_t)(h - 1) * W + w]);
        for (uint64_t i = 0; i < (uint64_t)H * W; ++i) xp[i] = (float)dp[i] * ebx2;
    }
    for (uint64_t k = 0; k < n_rec; ++k) {
        uint32_t key = rec[2 * k];
        if (key & 1u) xhat[key >> 1] = u2f(rec[2 * k + 1]);
    }
    for (uint64_t i = 0; i < n; ++i) if (fabsf(xhat[i]) <= eb) xhat[i] = 0.0f;
    free(d);
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Container                                                                  */
/* ------------------------------------------------------------------------- */
/*
 * All integers little-endian; sections start on 16-byte boundaries; padding is
 * zero.  Header, 128 bytes (u32 unless noted):
 *   0 magic  4 version(1)  8 status(0)  12 N  16 C  20 H  24 W  28 nbins
 *   32 chunk_syms  36 n_chunks  40 eb bits  44 2eb bits  48 r bits
 *   52 n_active  56 max_len  60 n_outlier_records
 *   64 nnz(u64)  72 payload_words(u64)  80 total_bytes(u64)
 *   88 off_len(u64)=128  96 off_chunk(u64)  104 off_outlier(u64)
 *   112 off_payload(u64)  120 n_value_records  124 zero
 * Sections: len[nbins] u8; chunk_off[n_chunks] u32 (word offset of each chunk in
 * the payload); outlier records (u32 key, u32 payload), ascending key;
 * payload[payload_words] u32.  total_bytes = off_payload + 4*payload_words.
 */
static uint64_t align16(uint64_t v) { return (v + 15u) & ~(uint64_t)15u; }

static void put32(uint8_t *p, uint32_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24); }
static void put64(uint8_t *p, uint64_t v) { put32(p, (uint32_t)v); put32(p + 4, (uint32_t)(v >> 32)); }
static uint32_t get32(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24); }
static uint64_t get64(const uint8_t *p) { return (uint64_t)get32(p) | ((uint64_t)get32(p + 4) << 32); }

/* Worst-case container size for a shape: every element escapes and is stored
 * verbatim, and the Huffman payload is bounded by 17 bits per symbol on average
 * (an optimal prefix code never averages more than log2(nbins) + 1 bits). */
uint64_t oracle_compress_bound(uint32_t N, uint32_t C, uint32_t H, uint32_t W,
                               uint32_t nbins, uint32_t chunk_syms) {
    uint64_t n;
    if (!shape_elems(N, C, H, W, &n) || !valid_nbins(nbins) || chunk_syms == 0) return 0;
    uint64_t n_chunks = (n + chunk_syms - 1u) / chunk_syms;
    uint64_t sz = ORC_HEADER_BYTES;
    sz = align16(sz + nbins);
    sz = align16(sz + 4u * n_chunks);
    sz = align16(sz + 8u * 2u * n);
    sz += 4u * ((17u * n + 31u) / 32u + n_chunks);
    return sz;
}

/*
 * A length table a caller brings along (codebook reuse, below) must describe a
 * code the decoder accepts: lengths 1..57, and either one active symbol of
 * length 1 or a complete prefix code (Kraft sum exactly 1).
 */
static int valid_given_lengths(const uint8_t *len, uint32_t nbins) {
    uint64_t kraft = 0;                      /* in units of 2^-57 */
    uint32_t active = 0;
    for (uint32_t s = 0; s < nbins; ++s) {
        if (!len[s]) continue;
        if (len[s] > 57u) return 0;
        ++active;
        kraft += 1ull << (57u - len[s]);
        if (kraft > (1ull << 57)) return 0;
    }
    if (active == 0) return 0;
    if (active == 1) return kraft == (1ull << 56);          /* one symbol: one bit per occurrence */
    return kraft == (1ull << 57);
}

/*
 * given == NULL: the pipeline of the paper (Sec. 4.1): the code book is built
 * from the histogram of this tensor.
 * given != NULL: code book reuse.  The paper refreshes its per-layer statistics
 * only every W iterations because they change slowly (Sec. 3.1); the same holds
 * for a layer's histogram, so a caller may keep the length table of an earlier
 * compression of the layer.  Steps 1-2 are unchanged; a quantisation code that
 * has no code word in the given table is treated exactly like a residual outside
 * the alphabet: it becomes the escape symbol 0 and its residual goes to the
 * outlier records.  If an escape is needed and the table has no code word for
 * the escape symbol either (the earlier tensor had none), the table cannot
 * represent this tensor: ORC_ERR_INVALID, and the caller compresses in full.
 * Steps 3-4 are skipped; canonical codes, encoding and the
 * container follow from the given lengths, which are stored in the container as
 * usual, so the decoder needs no change and the reconstruction is the one the
 * full pipeline gives.
 */
#define ORC_ZERO_CHUNKS 1u   /* container version 2: all-centre chunks take no words (see encode_impl) */
#define ORC_ZERO_FIRST 2u    /* zeros forced in the first quantisation step (see oracle_prequant_zero_first) */

static int compress_impl(const float *x, uint32_t N, uint32_t C, uint32_t H, uint32_t W,
                         float eb, uint32_t nbins, uint32_t chunk_syms, const uint8_t *given, uint32_t flags,
                         uint8_t *out, uint64_t capacity, uint64_t *used) {
    uint64_t n;
    if (!x || !out || !used || !valid_eb(eb) || !valid_nbins(nbins) || chunk_syms == 0 ||
        !shape_elems(N, C, H, W, &n)) return ORC_ERR_INVALID;
    if (given && !valid_given_lengths(given, nbins)) return ORC_ERR_INVALID;
    if (flags & ~(ORC_ZERO_CHUNKS | ORC_ZERO_FIRST)) return ORC_ERR_INVALID;
    float ebx2, r;
    oracle_constants(eb, &ebx2, &r);
    uint64_t n_chunks = (n + chunk_syms - 1u) / chunk_syms;
    int rc = ORC_OK;
    int32_t *q = (int32_t *)malloc((size_t)n * 4u);
    int32_t *delta = (int32_t *)malloc((size_t)n * 4u);
    uint8_t *vflag = (uint8_t *)malloc((size_t)n);
    uint16_t *codes = (uint16_t *)malloc((size_t)n * 2u);
    uint32_t *freq = (uint32_t *)malloc((size_t)nbins * 4u);
    uint8_t *len = (uint8_t *)malloc(nbins);
    uint64_t *code = (uint64_t *)malloc((size_t)nbins * 8u);
    uint32_t *chunk_off = (uint32_t *)malloc((size_t)n_chunks * 4u);
    if (!q || !delta || !vflag || !codes || !freq || !len || !code || !chunk_off) { rc = ORC_ERR_NOMEM; goto done; }
    uint64_t nnz = 0;
    if ((rc = prequant_impl(x, n, eb, (flags & ORC_ZERO_FIRST) != 0, q, vflag, &nnz)) != ORC_OK) goto done;
    if ((rc = oracle_predict_code(q, N, C, H, W, nbins, codes, delta)) != ORC_OK) goto done;
    if (given) {
        memcpy(len, given, nbins);
        for (uint64_t i = 0; i < n; ++i) {
            if (len[codes[i]] == 0) codes[i] = 0;             /* no code word: escape */
            if (codes[i] == 0 && len[0] == 0) { rc = ORC_ERR_INVALID; goto done; }
        }
    } else {
        if ((rc = oracle_histogram(codes, n, nbins, freq)) != ORC_OK) goto done;
        if ((rc = oracle_code_lengths(freq, nbins, len)) != ORC_OK) goto done;
    }
    if ((rc = oracle_canonical_codes(len, nbins, code)) != ORC_OK) goto done;

    uint64_t n_rec = 0, n_vrec = 0;
    for (uint64_t i = 0; i < n; ++i) { if (codes[i] == 0) ++n_rec; if (vflag[i]) { ++n_rec; ++n_vrec; } }
    uint32_t n_active = 0, max_len = 0;
    for (uint32_t s = 0; s < nbins; ++s) if (len[s]) { ++n_active; if (len[s] > max_len) max_len = len[s]; }

    uint64_t off_len = ORC_HEADER_BYTES;
    uint64_t off_chunk = align16(off_len + nbins);
    uint64_t off_outlier = align16(off_chunk + 4u * n_chunks);
    uint64_t off_payload = align16(off_outlier + 8u * n_rec);
    if (off_payload > capacity) { rc = ORC_ERR_CAPACITY; goto done; }
    uint64_t payload_cap_words = (capacity - off_payload) / 4u;
    memset(out, 0, (size_t)off_payload);
    uint64_t payload_words = 0;
    rc = encode_impl(codes, n, nbins, chunk_syms, len, code, (flags & ORC_ZERO_CHUNKS) != 0, chunk_off, n_chunks,
                     (uint32_t *)(void *)(out + off_payload), payload_cap_words, &payload_words);
    if (rc != ORC_OK) goto done;
    uint64_t total = off_payload + 4u * payload_words;

    put32(out + 0, ORC_MAGIC); put32(out + 4, (flags & ORC_ZERO_CHUNKS) ? 2u : 1u); put32(out + 8, 0u);
    put32(out + 12, N); put32(out + 16, C); put32(out + 20, H); put32(out + 24, W);
    put32(out + 28, nbins); put32(out + 32, chunk_syms); put32(out + 36, (uint32_t)n_chunks);
    put32(out + 40, f2u(eb)); put32(out + 44, f2u(ebx2)); put32(out + 48, f2u(r));
    put32(out + 52, n_active); put32(out + 56, max_len); put32(out + 60, (uint32_t)n_rec);
    put64(out + 64, nnz); put64(out + 72, payload_words); put64(out + 80, total);
    put64(out + 88, off_len); put64(out + 96, off_chunk); put64(out + 104, off_outlier);
    put64(out + 112, off_payload); put32(out + 120, (uint32_t)n_vrec); put32(out + 124, 0u);
    memcpy(out + off_len, len, nbins);
    for (uint64_t j = 0; j < n_chunks; ++j) put32(out + off_chunk + 4u * j, chunk_off[j]);
    {
        uint8_t *p = out + off_outlier;
        for (uint64_t i = 0; i < n; ++i) {
            if (codes[i] == 0) { put32(p, (uint32_t)(2u * i)); put32(p + 4, (uint32_t)delta[i]); p += 8; }
            if (vflag[i]) { put32(p, (uint32_t)(2u * i + 1u)); put32(p + 4, f2u(x[i])); p += 8; }
        }
    }
    *used = total;
done:
    free(q); free(delta); free(vflag); free(codes); free(freq); free(len); free(code); free(chunk_off);
    return rc;
}

int oracle_compress(const float *x, uint32_t N, uint32_t C, uint32_t H, uint32_t W,
                    float eb, uint32_t nbins, uint32_t chunk_syms,
                    uint8_t *out, uint64_t capacity, uint64_t *used) {
    return compress_impl(x, N, C, H, W, eb, nbins, chunk_syms, NULL, 0u, out, capacity, used);
}

/* The zero-handling variants: flags is a sum of ORC_ZERO_CHUNKS (1) and ORC_ZERO_FIRST (2). */
int oracle_compress_variant(const float *x, uint32_t N, uint32_t C, uint32_t H, uint32_t W,
                            float eb, uint32_t nbins, uint32_t chunk_syms, uint32_t flags,
                            uint8_t *out, uint64_t capacity, uint64_t *used) {
    return compress_impl(x, N, C, H, W, eb, nbins, chunk_syms, NULL, flags, out, capacity, used);
}

/* Compression with the length table of an earlier compression (see compress_impl). */
int oracle_compress_with_lengths(const float *x, uint32_t N, uint32_t C, uint32_t H, uint32_t W,
                                 float eb, uint32_t nbins, uint32_t chunk_syms, const uint8_t *given_len,
                                 uint8_t *out, uint64_t capacity, uint64_t *used) {
    if (!given_len) return ORC_ERR_INVALID;
    return compress_impl(x, N, C, H, W, eb, nbins, chunk_syms, given_len, 0u, out, capacity, used);
}

int oracle_decompress(const uint8_t *in, uint64_t bytes, float *out, uint64_t out_cap_elems,
                      uint32_t *shape_out /* N,C,H,W or NULL */) {
    if (!in || !out) return ORC_ERR_INVALID;
    if (bytes < ORC_HEADER_BYTES) return ORC_ERR_FORMAT;
    uint32_t version = get32(in + 4);
    if (get32(in + 0) != ORC_MAGIC || (version != 1u && version != 2u) || get32(in + 8) != 0u) return ORC_ERR_FORMAT;
    uint32_t N = get32(in + 12), C = get32(in + 16), H = get32(in + 20), W = get32(in + 24);
    uint32_t nbins = get32(in + 28), chunk_syms = get32(in + 32), n_chunks = get32(in + 36);
    float eb = u2f(get32(in + 40));
    uint32_t n_rec = get32(in + 60);
    uint64_t payload_words = get64(in + 72), total = get64(in + 80);
    uint64_t off_len = get64(in + 88), off_chunk = get64(in + 96), off_outlier = get64(in + 104), off_payload = get64(in + 112);
    uint64_t n;
    if (!shape_elems(N, C, H, W, &n) || !valid_nbins(nbins) || !valid_eb(eb) || chunk_syms == 0) return ORC_ERR_FORMAT;
    float ebx2, r;
    oracle_constants(eb, &ebx2, &r);
    if (f2u(ebx2) != get32(in + 44) || f2u(r) != get32(in + 48)) return ORC_ERR_FORMAT;
    if (n_chunks != (n + chunk_syms - 1u) / chunk_syms) return ORC_ERR_FORMAT;
    if (off_len != ORC_HEADER_BYTES || off_chunk != align16(off_len + nbins) ||
        off_outlier != align16(off_chunk + 4ull * n_chunks) ||
        off_payload != align16(off_outlier + 8ull * n_rec) ||
        total != off_payload + 4ull * payload_words || total > bytes) return ORC_ERR_FORMAT;
    if (n > out_cap_elems) return ORC_ERR_CAPACITY;
    int rc;
    uint16_t *codes = (uint16_t *)malloc((size_t)n * 2u);
    uint32_t *chunk_off = (uint32_t *)malloc((size_t)n_chunks * 4u);
    uint32_t *rec = (uint32_t *)malloc((size_t)n_rec * 8u + 8u);
    uint32_t *payload = (uint32_t *)malloc((size_t)payload_words * 4u + 4u);
    if (!codes || !chunk_off || !rec || !payload) { rc = ORC_ERR_NOMEM; goto done; }
    for (uint64_t j = 0; j < n_chunks; ++j) chunk_off[j] = get32(in + off_chunk + 4u * j);
    for (uint64_t k = 0; k < 2ull * n_rec; ++k) rec[k] = get32(in + off_outlier + 4u * k);
    for (uint64_t k = 0; k < payload_words; ++k) payload[k] = get32(in + off_payload + 4u * k);
    rc = decode_impl(in + off_len, nbins, version == 2u, chunk_off, payload, payload_words, n, chunk_syms, codes);
    if (rc != ORC_OK) goto done;
    rc = oracle_reconstruct(codes, rec, n_rec, N, C, H, W, nbins, eb, out);
    if (rc == ORC_OK && shape_out) { shape_out[0] = N; shape_out[1] = C; shape_out[2] = H; shape_out[3] = W; }
done:
    free(codes); free(chunk_off); free(rec); free(payload);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Adaptive error bound (Sec. 3.2 and Sec. 3.3)                               */
/* ------------------------------------------------------------------------- */
/*
 * sigma = sigma_frac * M (Sec. 3.2, sigma_frac = 0.01 by default), then
 * eb = sigma / (a * Lbar * sqrt(N * R)) (Sec. 3.3) with a = 0.32 (Sec. 5.2),
 * M the mean |momentum|, Lbar the mean |gradient of the loss| at the layer,
 * N the batch size and R the fraction of non-zero activations (Sec. 4.2).
 * All in fp64, rounded once to fp32, clamped to [eb_min, eb_max].  Lbar = 0 or
 * R = 0 (no error can reach the gradient) gives eb_max.
 */
int oracle_adapt_eb(double momentum_abs_mean, double loss_grad_mean, double nonzero_ratio,
                    uint32_t batch, double a, double sigma_frac, float eb_min, float eb_max,
                    float *eb_out) {
    if (!eb_out) return ORC_ERR_INVALID;
    if (!isfinite(momentum_abs_mean) || !isfinite(loss_grad_mean) || !isfinite(nonzero_ratio) ||
        !isfinite(a) || !isfinite(sigma_frac)) return ORC_ERR_INVALID;
    if (momentum_abs_mean < 0.0 || loss_grad_mean < 0.0 || nonzero_ratio < 0.0 || nonzero_ratio > 1.0 ||
        batch == 0 || !(a > 0.0) || !(sigma_frac > 0.0) || !(eb_min > 0.0f) || !(eb_max >= eb_min)) return ORC_ERR_INVALID;
    if (loss_grad_mean == 0.0 || nonzero_ratio == 0.0) { *eb_out = eb_max; return ORC_OK; }
    double sigma = sigma_frac * momentum_abs_mean;
    double eb = sigma / (a * loss_grad_mean * sqrt((double)batch * nonzero_ratio));
    float e = (float)eb;
    if (!(e >= eb_min)) e = eb_min;
    if (e > eb_max) e = eb_max;
    *eb_out = e;
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Controller glue (Sec. 3.1): a semi-online statistic and the active factor  */
/* ------------------------------------------------------------------------- */
/*
 * "Average value of the momentum" and "average gradient of the loss" (Sec. 3.1)
 * are taken as means of absolute values (a signed mean of either is about zero
 * and would give a zero error bound): sum of |x[i]| in fp64, in index order,
 * divided by n.
 */
int oracle_abs_mean(const float *x, uint64_t n, double *mean_out) {
    if (!x || !mean_out || n == 0) return ORC_ERR_INVALID;
    double sum = 0.0;
    for (uint64_t i = 0; i < n; ++i) sum += fabs((double)x[i]);
    *mean_out = sum / (double)n;
    return ORC_OK;
}

/*
 * Active factor W (Sec. 3.1): the semi-online parameters are collected, and the
 * error bounds re-estimated, every W iterations; W starts at its default (1000).
 * After a re-estimation the largest change of a layer's bound since the
 * previous one is looked at, as a ratio >= 1 in either direction: above 2, W
 * is halved (never below 1); otherwise the bounds have settled and W returns to
 * its default.  state[0] = default, state[1] = W, state[2] = iterations since
 * the last collection.
 */
int oracle_controller_init(uint32_t *state, uint32_t w_default) {
    if (!state) return ORC_ERR_INVALID;
    state[0] = w_default ? w_default : 1000u;
    state[1] = state[0];
    state[2] = 0;
    return ORC_OK;
}

/* One iteration has passed; *collect = 1 in every W-th one. */
int oracle_controller_tick(uint32_t *state, int *collect) {
    if (!state || !collect || state[1] == 0) return ORC_ERR_INVALID;
    state[2] += 1u;
    *collect = 0;
    if (state[2] >= state[1]) { state[2] = 0; *collect = 1; }
    return ORC_OK;
}

int oracle_controller_update(uint32_t *state, const float *eb_old, const float *eb_new, uint32_t n_layers) {
    if (!state || !eb_old || !eb_new || n_layers == 0 || state[1] == 0) return ORC_ERR_INVALID;
    double worst = 1.0;
    for (uint32_t l = 0; l < n_layers; ++l) {
        double a = (double)eb_old[l], b = (double)eb_new[l];
        if (!(a > 0.0) || !(b > 0.0) || !isfinite(a) || !isfinite(b)) return ORC_ERR_INVALID;
        double ratio = a > b ? a / b : b / a;
        if (ratio > worst) worst = ratio;
    }
    if (worst > 2.0) state[1] = state[1] > 1u ? state[1] / 2u : 1u;
    else state[1] = state[0];
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* 16-bit activations (an extension; the paper trains in fp32).  The codec     */
/* stays the fp32 one of Sec. 4.1: a 16-bit input is widened to fp32 (exact    */
/* for both formats) and compressed as such; a 16-bit output is the fp32       */
/* reconstruction rounded to the nearest value of the format, ties to even.    */
/* Both conversions are written out from the definition of a binary            */
/* floating-point format with p significand bits (implicit bit included) and   */
/* exponent range [emin, emax]: binary16 p = 11, emin = -14, emax = 15;        */
/* bfloat16 p = 8, emin = -126, emax = 127.                                    */
/* Pins: all 65536 binary16 patterns and random / edge fp32 values against     */
/* numpy's float16, bfloat16 against torch's CPU conversion, hand cases        */
/* (ties, overflow to infinity, subnormals, signed zero).                      */
/* ------------------------------------------------------------------------- */
static int fmt_of(int kind, int *p, int *emin, int *emax) {
    if (kind == 1) { *p = 11; *emin = -14; *emax = 15; return 1; }
    if (kind == 2) { *p = 8; *emin = -126; *emax = 127; return 1; }
    return 0;
}

/* value of the 16-bit pattern h */
static float widen_one(uint16_t h, int p, int emin, int emax) {
    const int ebits = 16 - p;                       /* 1 sign bit + ebits + (p - 1) fraction bits */
    const uint32_t frac = h & ((1u << (p - 1)) - 1u);
    const uint32_t ef = ((uint32_t)h >> (p - 1)) & ((1u << ebits) - 1u);
    const double sign = (h & 0x8000u) ? -1.0 : 1.0;
    if (ef == (1u << ebits) - 1u) return (float)(frac ? NAN : sign * INFINITY);
    if (ef == 0) return (float)(sign * ldexp((double)frac, emin - (p - 1)));           /* subnormal or zero */
    (void)emax;
    return (float)(sign * ldexp((double)(frac | (1u << (p - 1))), (int)ef - (emax) - (p - 1)));  /* bias = emax */
}

/* nearest value of the format to x, ties to even, as its bit pattern */
static uint16_t narrow_one(float x, int p, int emin, int emax) {
    const int ebits = 16 - p;
    const uint16_t sign = signbit(x) ? 0x8000u : 0u;
    const uint16_t inf = (uint16_t)(((1u << ebits) - 1u) << (p - 1));
    if (isnan(x)) return (uint16_t)(sign | inf | (1u << (p - 2)));
    double a = fabs((double)x);
    if (isinf(x)) return (uint16_t)(sign | inf);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                             /* a = m * 2^e, 0.5 <= m < 1: the leading bit has weight 2^(e-1) */
    int E = e - 1;
    if (E < emin) E = emin;                         /* subnormal range: fixed spacing */
    const double quantum = ldexp(1.0, E - (p - 1));
    const double v = nearbyint(a / quantum) * quantum;   /* round-to-nearest-even is the default mode; the scaling is exact */
    if (v >= ldexp(1.0, emax + 1)) return (uint16_t)(sign | inf);
    if (v == 0.0) return sign;
    (void)frexp(v, &e);
    const int E2 = e - 1;
    if (E2 < emin) return (uint16_t)(sign | (uint16_t)(v / ldexp(1.0, emin - (p - 1))));
    const uint32_t sig = (uint32_t)(v / ldexp(1.0, E2 - (p - 1)));      /* p bits, leading one set */
    return (uint16_t)(sign | (uint32_t)((E2 + emax) << (p - 1)) | (sig & ((1u << (p - 1)) - 1u)));
}

/* kind: 1 binary16, 2 bfloat16 */
int oracle_widen16(const uint16_t *in, int kind, float *out, uint64_t n) {
    int p, emin, emax;
    if (!in || !out || !fmt_of(kind, &p, &emin, &emax)) return ORC_ERR_INVALID;
    for (uint64_t i = 0; i < n; ++i) out[i] = widen_one(in[i], p, emin, emax);
    return ORC_OK;
}

int oracle_narrow16(const float *in, int kind, uint16_t *out, uint64_t n) {
    int p, emin, emax;
    if (!in || !out || !fmt_of(kind, &p, &emin, &emax)) return ORC_ERR_INVALID;
    for (uint64_t i = 0; i < n; ++i) out[i] = narrow_one(in[i], p, emin, emax);
    return ORC_OK;
}
