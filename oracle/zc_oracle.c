/*
 * zc_oracle.c -- CPU oracle for the field-split Huffman tensor codec ("ZC1").
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded
 * statement of what the codec computes, written to be checked by eye against
 * the paper (Heilper & Singer, "Lossless Compression of Neural Network
 * Components", 2025) and against the container definition below.  It shares no
 * code with the HIP library and must never be called from the product path;
 * only tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What the paper fixes (and where):
 *   - every value is split into its exponent bits and its sign+mantissa bits
 *     and the two are coded as independent streams        (Sec. 3.1, 3.2, Fig. 5)
 *   - BF16 = 1 sign, 8 exponent, 7 mantissa bits           (Sec. 3.1)
 *   - FP8 E4M3 = 1 sign, 4 exponent, 3 mantissa bits       (Sec. 3.2, Fig. 1)
 *   - FP4 = E2M1 elements plus a shared per-block scale; the scale stream is
 *     the compressible part                                (Sec. 3.4, 4.4)
 *   - a checkpoint delta is the bitwise XOR of two BF16 tensors, split and
 *     coded like any other tensor                          (Sec. 3.1, 4.1)
 *   - each stream is Huffman coded; a stream that does not compress may be
 *     stored as is                                         (Sec. 3.1, 4.3)
 *   - one code per tensor, data cut into fixed-size chunks that decode
 *     independently (random access, parallel decode)       (Sec. 3.1, Sec. 4)
 *   - the result is lossless                               (Sec. 1, 2.2)
 *
 * What the paper leaves open and this oracle therefore DEFINES (each reading
 * is listed in the design document): symbol layout inside a field, the
 * Huffman variant and its tie-breaks (length-limited package-merge, canonical
 * code assignment), the stream layout inside a chunk, and the container.
 *
 * Parity pins (tests/test_oracle_*.py): hand-worked field splits, exhaustive
 * split/rebuild identity, numpy.bincount, Kraft equality, entropy bounds,
 * brute-force optimal codes on <= 8 symbols, textbook heap Huffman cost,
 * hand-worked code tables and streams, an independent bit-by-bit reader for
 * the one-lane case, chunk independence, exact round trips; for the statistics
 * (tests/test_oracle_stats.py) hand-made fields with exact entropies and
 * -sum p log2 p recomputed with numpy from numpy.bincount of the symbols.
 * Parity unpinned: the ratios the paper reports on real checkpoints (the data
 * is not available); they are quoted as context only.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

/* ------------------------------------------------------------------ formats */

/* Formats 4 and 5 hold the same elements and the same two (three) fields as 2 and 3, but code the
 * field values in byte-sized groups (Sec. 3.2, Fig. 7: FP8 exponents and sign+mantissa values
 * paired into bytes; Sec. 3.4: four 2-bit FP4 values per byte): one Huffman symbol = one byte of
 * the packed field array = 2 (FP8) or 4 (FP4) consecutive field values, first value in the low bits. */
/* Format 6 is NVFP4 (Sec. 3.4): the E2M1 elements of format 3 with one FP8 (E4M3) scale byte per 16
 * elements instead of one E8M0 byte per 32; the scale bytes are coded as 8-bit symbols like the E8M0 ones. */
/* Format 7 is the other FP8 variant of Sec. 3.2, E5M2 (s eeeee mm): a 5-bit exponent and a 3-bit
 * sign+mantissa value per element, each coded as a symbol of its own that is held in 8 bits (alphabets of
 * 256 of which 32 and 8 can occur), so that a lane's run of 16 elements is 16 symbols in both fields. */
enum { ZCO_BF16 = 1, ZCO_FP8_E4M3 = 2, ZCO_FP4_E2M1_MX = 3, ZCO_FP8_E4M3_BYTES = 4, ZCO_FP4_E2M1_MX_BYTES = 5, ZCO_FP4_E2M1_NV = 6,
       ZCO_FP8_E5M2 = 7 };
enum { ZCO_MODE_EMPTY = 0, ZCO_MODE_HUFF = 1, ZCO_MODE_RAW = 2, ZCO_MODE_CONST = 3 };
enum { ZCO_POLICY_HUFF_ALL = 0, ZCO_POLICY_AUTO = 1 };
enum { ZCO_OK = 0, ZCO_ERR_ARG = 1, ZCO_ERR_UNSUPPORTED = 2, ZCO_ERR_SMALL = 3, ZCO_ERR_CORRUPT = 4 };

typedef struct {
    uint32_t format;
    uint32_t chunk_bytes;        /* bytes of element data per chunk */
    uint32_t max_code_len[3];    /* per field; 0 = default */
    uint32_t streams_per_chunk;  /* S; 0 = 64 */
    uint32_t policy;
    uint32_t payload_order;      /* 0: the streams of field 0 first, then field 1, ...; 1: the last field first */
} zco_params;

/* element format of a (possibly byte-grouped) format, and field values per coded symbol */
static int base_format(int format)
{
    if (format == ZCO_FP4_E2M1_NV) return ZCO_FP4_E2M1_MX;        /* same elements, other scales */
    return format == ZCO_FP8_E4M3_BYTES ? ZCO_FP8_E4M3 : format == ZCO_FP4_E2M1_MX_BYTES ? ZCO_FP4_E2M1_MX : format;
}

/* elements that share one scale byte (0: the format has no scales) */
static int scale_block(int format)
{
    return format == ZCO_FP4_E2M1_NV ? 16 : (format == ZCO_FP4_E2M1_MX || format == ZCO_FP4_E2M1_MX_BYTES) ? 32 : 0;
}

static int group_of(int format)
{
    return format == ZCO_FP8_E4M3_BYTES ? 2 : format == ZCO_FP4_E2M1_MX_BYTES ? 4 : 1;
}

static int elem_bits(int format)
{
    format = base_format(format);
    return format == ZCO_BF16 ? 16 : (format == ZCO_FP8_E4M3 || format == ZCO_FP8_E5M2) ? 8 : format == ZCO_FP4_E2M1_MX ? 4 : 0;
}

int zco_num_fields(int format)
{
    format = base_format(format);
    return format == ZCO_FP4_E2M1_MX ? 3 : (format == ZCO_BF16 || format == ZCO_FP8_E4M3 || format == ZCO_FP8_E5M2) ? 2 : 0;
}

/* width of one field value of field f: field 0 = exponent, 1 = sign+mantissa, 2 = block scale */
static int value_bits(int format, int f)
{
    format = base_format(format);
    if (format == ZCO_BF16) return 8;
    if (format == ZCO_FP8_E4M3) return 4;
    if (format == ZCO_FP8_E5M2) return f == 0 ? 5 : 3;
    if (format == ZCO_FP4_E2M1_MX) return f == 2 ? 8 : 2;
    return 0;
}

/* width of one coded symbol of field f */
int zco_sym_bits(int format, int f)
{
    if (!elem_bits(format)) return 0;
    if (format == ZCO_FP8_E5M2) return 8;                      /* 5- and 3-bit values held in 8-bit symbols */
    return f == 2 ? 8 : value_bits(format, f) * group_of(format);
}

/* symbols that make up one 16-byte run of the field's plain array */
static int run_len(int format, int f)
{
    if (f == 2) return 16;                                     /* 16 scale bytes */
    return 128 / elem_bits(format) / group_of(format);         /* 16 bytes of elements */
}

static uint64_t num_symbols(int format, int f, uint64_t n_elems)
{
    if (f == 2) return n_elems / (uint64_t)scale_block(format);   /* one scale byte per block of elements */
    return (n_elems + (uint64_t)group_of(format) - 1) / (uint64_t)group_of(format);
}

/* ---------------------------------------------------- field split / rebuild */
/* Sec. 3.1 / 3.2 / 3.4: the exponent bits form one symbol, the sign bit placed
 * above the mantissa bits forms the other.  Values are never interpreted. */

/* element i of the tensor as an unsigned integer (FP4: element 2i is the low nibble) */
static unsigned load_elem(int format, const uint8_t *p, uint64_t i)
{
    format = base_format(format);
    if (format == ZCO_BF16) return (unsigned)p[2 * i] | ((unsigned)p[2 * i + 1] << 8);
    if (format == ZCO_FP8_E4M3 || format == ZCO_FP8_E5M2) return p[i];
    return (i & 1) ? (p[i / 2] >> 4) : (p[i / 2] & 0xF);
}

static void store_elem(int format, uint8_t *p, uint64_t i, unsigned x)
{
    format = base_format(format);
    if (format == ZCO_BF16) { p[2 * i] = (uint8_t)(x & 0xFF); p[2 * i + 1] = (uint8_t)(x >> 8); }
    else if (format == ZCO_FP8_E4M3 || format == ZCO_FP8_E5M2) p[i] = (uint8_t)x;
    else if (i & 1) p[i / 2] = (uint8_t)((p[i / 2] & 0x0F) | (x << 4));
    else p[i / 2] = (uint8_t)((p[i / 2] & 0xF0) | (x & 0xF));
}

unsigned zco_exponent_of(int format, unsigned x)
{
    format = base_format(format);
    if (format == ZCO_BF16) return (x >> 7) & 0xFF;        /* s eeeeeeee mmmmmmm */
    if (format == ZCO_FP8_E4M3) return (x >> 3) & 0xF;     /* s eeee mmm */
    if (format == ZCO_FP8_E5M2) return (x >> 2) & 0x1F;    /* s eeeee mm */
    return (x >> 1) & 0x3;                                 /* s ee m */
}

unsigned zco_signmant_of(int format, unsigned x)
{
    format = base_format(format);
    if (format == ZCO_BF16) return ((x >> 15) << 7) | (x & 0x7F);
    if (format == ZCO_FP8_E4M3) return ((x >> 7) << 3) | (x & 0x7);
    if (format == ZCO_FP8_E5M2) return ((x >> 7) << 2) | (x & 0x3);
    return ((x >> 3) << 1) | (x & 0x1);
}

unsigned zco_rebuild(int format, unsigned e, unsigned sm)
{
    format = base_format(format);
    if (format == ZCO_BF16) return ((sm >> 7) << 15) | (e << 7) | (sm & 0x7F);
    if (format == ZCO_FP8_E4M3) return ((sm >> 3) << 7) | (e << 3) | (sm & 0x7);
    if (format == ZCO_FP8_E5M2) return ((sm >> 2) << 7) | (e << 2) | (sm & 0x3);
    return ((sm >> 1) << 3) | (e << 1) | (sm & 0x1);
}

/* Split a tensor into one-symbol-per-byte arrays.  base (may be NULL) is XORed
 * onto the bit patterns first (Sec. 3.1, 4.1: delta of consecutive checkpoints). */
void zco_split(int format, const uint8_t *src, const uint8_t *base, uint64_t n_elems,
               uint8_t *exp_out, uint8_t *sm_out)
{
    for (uint64_t i = 0; i < n_elems; i++) {
        unsigned x = load_elem(format, src, i);
        if (base) x ^= load_elem(format, base, i);
        exp_out[i] = (uint8_t)zco_exponent_of(format, x);
        sm_out[i] = (uint8_t)zco_signmant_of(format, x);
    }
}

void zco_join(int format, const uint8_t *exp_in, const uint8_t *sm_in, const uint8_t *base,
              uint64_t n_elems, uint8_t *dst)
{
    for (uint64_t i = 0; i < n_elems; i++) {
        unsigned x = zco_rebuild(format, exp_in[i], sm_in[i]);
        if (base) x ^= load_elem(format, base, i);
        store_elem(format, dst, i, x);
    }
}

/* Coded symbols of field f (0 or 1) from its field values (one per byte, as zco_split leaves them):
 * symbol j = values g*j .. g*j+g-1, the first in the low bits; values past the end count as 0. */
void zco_group_values(int format, int f, const uint8_t *values, uint64_t n_elems, uint8_t *syms)
{
    int g = group_of(format), vb = value_bits(format, f);
    uint64_t ns = num_symbols(format, f, n_elems);
    for (uint64_t j = 0; j < ns; j++) {
        unsigned s = 0;
        for (int k = 0; k < g; k++)
            if (g * j + (uint64_t)k < n_elems) s |= (unsigned)values[g * j + (uint64_t)k] << (k * vb);
        syms[j] = (uint8_t)s;
    }
}

void zco_ungroup_symbols(int format, int f, const uint8_t *syms, uint64_t n_elems, uint8_t *values)
{
    int g = group_of(format), vb = value_bits(format, f);
    for (uint64_t i = 0; i < n_elems; i++)
        values[i] = (uint8_t)((syms[i / (uint64_t)g] >> ((int)(i % (uint64_t)g) * vb)) & ((1u << vb) - 1));
}

void zco_histogram(const uint8_t *syms, uint64_t n, uint64_t *hist256)
{
    memset(hist256, 0, 256 * sizeof(uint64_t));
    for (uint64_t i = 0; i < n; i++) hist256[syms[i]]++;
}

/* ------------------------------------------- Huffman code lengths (limit L) */
/*
 * Length-limited optimal prefix code by the package-merge (coin collector)
 * construction of Larmore and Hirschberg, stated with explicit membership so
 * that it can be read as the definition:
 *
 *   leaves  = the symbols with freq > 0, ordered by (freq, symbol) ascending
 *   row[L]  = leaves
 *   row[d]  = merge(leaves, packages(row[d+1]))   for d = L-1 .. 1
 *             packages() joins items 2k and 2k+1 of a row (an odd last item is
 *             dropped); merge() orders by weight, a leaf before a package of
 *             equal weight, each side keeping its own order
 *   answer  = the first 2*(#leaves) - 2 items of row[1]; the code length of a
 *             symbol is the number of those items that contain its leaf.
 *
 * The tie rules make the lengths unique.  One active symbol gets length 1
 * here; the container stores such a field in CONST mode and never uses it.
 * Returns 0, or -1 if 2^L < number of active symbols.
 */
typedef struct { uint64_t w; uint16_t cnt[256]; int is_leaf; } pm_item;

int zco_code_lengths(const uint64_t *hist, int alphabet, int L, uint8_t *len_out)
{
    int sym[256], n = 0;
    memset(len_out, 0, (size_t)alphabet);
    for (int v = 0; v < alphabet; v++) if (hist[v]) sym[n++] = v;
    if (n == 0) return 0;
    if (n == 1) { len_out[sym[0]] = 1; return 0; }
    if (L < 1 || L > 16 || (1 << L) < n) return -1;
    /* insertion sort by (freq, symbol); sym[] is already ascending in symbol */
    for (int i = 1; i < n; i++) {
        int s = sym[i], j = i;
        while (j > 0 && hist[sym[j - 1]] > hist[s]) { sym[j] = sym[j - 1]; j--; }
        sym[j] = s;
    }
    pm_item *leaves = calloc((size_t)n, sizeof(pm_item));
    pm_item *row = calloc((size_t)(2 * n), sizeof(pm_item));
    pm_item *pk = calloc((size_t)n, sizeof(pm_item));
    pm_item *nxt = calloc((size_t)(2 * n), sizeof(pm_item));
    for (int i = 0; i < n; i++) { leaves[i].w = hist[sym[i]]; leaves[i].cnt[sym[i]] = 1; leaves[i].is_leaf = 1; }
    int row_n = n;
    memcpy(row, leaves, (size_t)n * sizeof(pm_item));
    for (int d = L - 1; d >= 1; d--) {
        int pk_n = row_n / 2;
        for (int k = 0; k < pk_n; k++) {
            pk[k].w = row[2 * k].w + row[2 * k + 1].w;
            pk[k].is_leaf = 0;
            for (int v = 0; v < 256; v++) pk[k].cnt[v] = (uint16_t)(row[2 * k].cnt[v] + row[2 * k + 1].cnt[v]);
        }
        int a = 0, b = 0, m = 0;
        while (a < n || b < pk_n) {
            if (b >= pk_n || (a < n && leaves[a].w <= pk[b].w)) nxt[m++] = leaves[a++];
            else nxt[m++] = pk[b++];
        }
        pm_item *t = row; row = nxt; nxt = t;
        row_n = m;
    }
    for (int i = 0; i < 2 * n - 2; i++)
        for (int v = 0; v < alphabet; v++) len_out[v] = (uint8_t)(len_out[v] + row[i].cnt[v]);
    free(leaves); free(row); free(pk); free(nxt);
    return 0;
}

/* Canonical code values: symbols ordered by (length, symbol); the first code is
 * 0; each next code is (previous + 1) shifted left by the growth in length. */
void zco_canonical_codes(const uint8_t *len, int alphabet, uint16_t *code_out)
{
    unsigned code = 0;
    int prev_len = 0, first = 1;
    memset(code_out, 0, (size_t)alphabet * sizeof(uint16_t));
    for (int l = 1; l <= 16; l++)
        for (int v = 0; v < alphabet; v++)
            if (len[v] == l) {
                if (first) { code = 0; first = 0; }
                else code = (code + 1) << (l - prev_len);
                prev_len = l;
                code_out[v] = (uint16_t)code;
            }
}

/* ------------------------------------------------------ lane-interleaved stream */
/*
 * One (chunk, field) in HUFF mode.  The n symbols of the chunk are dealt to S
 * lanes in runs of G: symbol j belongs to lane (j / G) mod S, and a lane keeps
 * its symbols in increasing j.  A lane's code words, each written most
 * significant bit first, form one bit string; bit i of that string is bit
 * (i mod 32) of the lane's 32-bit word number i / 32; bits past the end are 0.
 *
 * The order of the words in the stream is the order in which this decoder asks
 * for them.  Every lane holds a 64-bit buffer (next bit = bit 0) with k valid
 * bits, k = 0 at the start.  For t = 0, 1, 2, ...: a lane is active while it
 * still owns a t-th symbol.  If t is a multiple of the refill period r, every
 * active lane with k <= 32, in ascending lane order, takes the next
 * little-endian u32 of the stream into bits k..k+31 of its buffer.  Then every
 * active lane decodes one symbol.  r = min(G, largest power of two <= 32/Lmax),
 * Lmax being the longest code of the field's table, so at least r*Lmax bits
 * are valid after each refill step.  The stream is the words taken, followed
 * by zero bytes up to a multiple of 16.
 */
static int refill_period(int G, int lmax)
{
    int r = 1;
    if (lmax < 1) lmax = 1;
    while (2 * r * lmax <= 32) r *= 2;
    return r < G ? r : G;
}

static uint64_t lane_symbol_count(uint64_t n, int G, int S, int s)
{
    uint64_t cnt = 0, runs = (n + (uint64_t)G - 1) / (uint64_t)G;
    for (uint64_t q = (uint64_t)s; q < runs; q += (uint64_t)S) {
        uint64_t lo = q * (uint64_t)G, hi = lo + (uint64_t)G;
        cnt += (hi <= n ? hi : n) - lo;
    }
    return cnt;
}

/* position in the chunk of the t-th symbol of lane s */
static uint64_t lane_symbol_index(uint64_t t, int G, int S, int s)
{
    return ((t / (uint64_t)G) * (uint64_t)S + (uint64_t)s) * (uint64_t)G + t % (uint64_t)G;
}

/* Encoder: builds every lane's bit string, then replays the decoder's requests.
 * out must have room for zco_stream_bound(n, S, lmax) bytes.  Returns bytes written. */
uint64_t zco_stream_bound(uint64_t n, int S, int lmax)
{
    return (n * (uint64_t)lmax + 31) / 32 * 4 + (uint64_t)S * 12 + 16;
}

uint64_t zco_encode_stream(const uint8_t *syms, uint64_t n, const uint8_t *len, const uint16_t *code,
                           int lmax, int G, int S, uint8_t *out)
{
    int r = refill_period(G, lmax);
    uint32_t **words = calloc((size_t)S, sizeof(uint32_t *));
    uint64_t *cnt = calloc((size_t)S, sizeof(uint64_t));
    uint64_t *nbits = calloc((size_t)S, sizeof(uint64_t));
    uint64_t *taken = calloc((size_t)S, sizeof(uint64_t));      /* words handed out */
    uint64_t *used = calloc((size_t)S, sizeof(uint64_t));       /* bits decoded so far */
    uint64_t max_cnt = 0, pos = 0;
    for (int s = 0; s < S; s++) {
        cnt[s] = lane_symbol_count(n, G, S, s);
        if (cnt[s] > max_cnt) max_cnt = cnt[s];
        words[s] = calloc((size_t)(cnt[s] * (uint64_t)lmax / 32 + 4), sizeof(uint32_t));
        for (uint64_t t = 0; t < cnt[s]; t++) {
            unsigned v = syms[lane_symbol_index(t, G, S, s)];
            for (int b = len[v] - 1; b >= 0; b--) {            /* most significant code bit first */
                if ((code[v] >> b) & 1) words[s][nbits[s] / 32] |= (uint32_t)1 << (nbits[s] % 32);
                nbits[s]++;
            }
        }
    }
    for (uint64_t t = 0; t < max_cnt; t++) {
        if (t % (uint64_t)r == 0)
            for (int s = 0; s < S; s++)
                if (t < cnt[s] && 32 * taken[s] - used[s] <= 32) {     /* k <= 32 */
                    uint32_t w = words[s][taken[s]++];
                    out[pos++] = (uint8_t)w; out[pos++] = (uint8_t)(w >> 8);
                    out[pos++] = (uint8_t)(w >> 16); out[pos++] = (uint8_t)(w >> 24);
                }
        for (int s = 0; s < S; s++)
            if (t < cnt[s]) used[s] += len[syms[lane_symbol_index(t, G, S, s)]];
    }
    while (pos % 16) out[pos++] = 0;
    for (int s = 0; s < S; s++) free(words[s]);
    free(words); free(cnt); free(nbits); free(taken); free(used);
    return pos;
}

/* canonical decoding tables: for each length, the first code value, how many
 * codes have that length, and where their symbols start in the sorted list */
typedef struct { unsigned first[17], count[17], start[17]; uint8_t sorted[256]; int lmax; } dec_table;

static int build_dec_table(const uint8_t *len, int alphabet, dec_table *d)
{
    unsigned code = 0, idx = 0;
    uint64_t kraft = 0;
    memset(d, 0, sizeof(*d));
    for (int v = 0; v < alphabet; v++) {
        if (len[v] > 16) return -1;
        if (len[v]) { d->count[len[v]]++; kraft += (uint64_t)1 << (16 - len[v]); if (len[v] > d->lmax) d->lmax = len[v]; }
    }
    if (kraft != 65536) return -1;           /* a HUFF table must be complete */
    for (int l = 1; l <= 16; l++) {
        code <<= 1;
        d->first[l] = code; d->start[l] = idx;
        for (int v = 0; v < alphabet; v++) if (len[v] == l) d->sorted[idx++] = (uint8_t)v;
        code += d->count[l];
    }
    return 0;
}

/* Decoder: the definition above, literally.  Returns bytes consumed (with the
 * padding), or 0 on a malformed stream (ran past avail, or no code matched). */
uint64_t zco_decode_stream(const uint8_t *in, uint64_t avail, uint64_t n, const uint8_t *len, int alphabet,
                           int G, int S, uint8_t *syms_out)
{
    dec_table d;
    if (build_dec_table(len, alphabet, &d)) return 0;
    int r = refill_period(G, d.lmax);
    uint64_t *buf = calloc((size_t)S, sizeof(uint64_t));
    int *k = calloc((size_t)S, sizeof(int));
    uint64_t *cnt = calloc((size_t)S, sizeof(uint64_t));
    uint64_t max_cnt = 0, pos = 0;
    int bad = 0;
    for (int s = 0; s < S; s++) { cnt[s] = lane_symbol_count(n, G, S, s); if (cnt[s] > max_cnt) max_cnt = cnt[s]; }
    for (uint64_t t = 0; t < max_cnt && !bad; t++) {
        if (t % (uint64_t)r == 0)
            for (int s = 0; s < S; s++)
                if (t < cnt[s] && k[s] <= 32) {
                    if (pos + 4 > avail) { bad = 1; break; }
                    uint64_t w = (uint64_t)in[pos] | ((uint64_t)in[pos + 1] << 8) | ((uint64_t)in[pos + 2] << 16) | ((uint64_t)in[pos + 3] << 24);
                    pos += 4;
                    buf[s] |= w << k[s];
                    k[s] += 32;
                }
        for (int s = 0; s < S && !bad; s++)
            if (t < cnt[s]) {
                unsigned code = 0;
                int l, found = 0;
                for (l = 1; l <= d.lmax; l++) {
                    code = (code << 1) | (unsigned)(buf[s] & 1);
                    buf[s] >>= 1; k[s]--;
                    if (code >= d.first[l] && code - d.first[l] < d.count[l]) {
                        syms_out[lane_symbol_index(t, G, S, s)] = d.sorted[d.start[l] + code - d.first[l]];
                        found = 1;
                        break;
                    }
                }
                if (!found || k[s] < 0) bad = 1;
            }
    }
    while (pos % 16) pos++;
    if (pos > avail) bad = 1;
    free(buf); free(k); free(cnt);
    return bad ? 0 : pos;
}

/* RAW mode: the symbols of the chunk in element order, sym_bits each, symbol j
 * occupying bits j*sym_bits.. of a little-endian bit string (bit i = bit i%8 of
 * byte i/8), zero padded to a multiple of 16 bytes. */
static uint64_t raw_stream_bytes(uint64_t n, int sym_bits)
{
    uint64_t b = (n * (uint64_t)sym_bits + 7) / 8;
    return (b + 15) / 16 * 16;
}

static uint64_t encode_raw(const uint8_t *syms, uint64_t n, int sym_bits, uint8_t *out)
{
    uint64_t bytes = raw_stream_bytes(n, sym_bits);
    memset(out, 0, (size_t)bytes);
    for (uint64_t j = 0; j < n; j++)
        for (int b = 0; b < sym_bits; b++)
            if ((syms[j] >> b) & 1) { uint64_t i = j * (uint64_t)sym_bits + (uint64_t)b; out[i / 8] |= (uint8_t)(1u << (i % 8)); }
    return bytes;
}

static void decode_raw(const uint8_t *in, uint64_t n, int sym_bits, uint8_t *syms_out)
{
    for (uint64_t j = 0; j < n; j++) {
        unsigned v = 0;
        for (int b = 0; b < sym_bits; b++) { uint64_t i = j * (uint64_t)sym_bits + (uint64_t)b; v |= (unsigned)((in[i / 8] >> (i % 8)) & 1) << b; }
        syms_out[j] = (uint8_t)v;
    }
}

/* --------------------------------------------------------------- container */
/*
 * "ZC1" container, little-endian, every section starting on a 16-byte boundary:
 *
 *   header (64 bytes)
 *      0  u32  magic 0x0031435A ("ZC1\0")
 *      4  u16  version = 1
 *      6  u8   format          7  u8  policy
 *      8  u8   S (lanes)       9  u8  number of fields
 *     10  u8   flags (bit 0: XOR delta against a base tensor; bit 1: payload in reverse field order)
 *     11  u8   0
 *     12  u32  chunk_bytes
 *     16  u64  n_elems
 *     24  u32  n_chunks       28  u32  0
 *     32  3 x { u8 mode, u8 sym_bits, u8 Lmax, u8 const_symbol }
 *     44  u32  0
 *     48  u64  total container bytes
 *     56  u64  payload offset
 *   per field: code-length table, 2^sym_bits bytes (0 = symbol absent; all 0
 *      unless mode = HUFF), padded to 16
 *   per field: chunk index, n_chunks + 1 u32 offsets in 16-byte units from the
 *      payload start, padded to 16.  Field-major: all streams of field 0, then
 *      field 1, ...; the first offset of a field equals the last of the one before.
 *      With flag bit 1 the fields follow each other in the payload from the last
 *      to the first (tables and indices stay where they are).  The paper leaves
 *      the arrangement of the compressed streams open (Sec. 3.1 asks for blocks
 *      that can be reached at random); the reverse order puts a sign+mantissa
 *      field of fixed stream size in front, so that where an exponent stream goes
 *      depends only on the exponent streams of the chunks before it (Sec. 5.2:
 *      K/V pages are compressed on the critical path, in one pass over them).
 *   payload: the (field, chunk) streams back to back.
 */
#define ZCO_MAGIC 0x0031435Au
#define ZCO_HEADER_BYTES 64

static uint64_t pad16(uint64_t x) { return (x + 15) / 16 * 16; }
static void put32(uint8_t *p, uint32_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24); }
static void put64(uint8_t *p, uint64_t v) { put32(p, (uint32_t)v); put32(p + 4, (uint32_t)(v >> 32)); }
static uint32_t get32(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24); }
static uint64_t get64(const uint8_t *p) { return (uint64_t)get32(p) | ((uint64_t)get32(p + 4) << 32); }

static int check_params(const zco_params *p, uint64_t n_elems, int *S)
{
    int eb = elem_bits((int)p->format);
    if (!eb) return ZCO_ERR_UNSUPPORTED;
    *S = p->streams_per_chunk ? (int)p->streams_per_chunk : 64;
    if (*S != 1 && *S != 2 && *S != 4 && *S != 8 && *S != 16 && *S != 32 && *S != 64) return ZCO_ERR_ARG;
    if (p->chunk_bytes == 0 || p->chunk_bytes % 16) return ZCO_ERR_ARG;
    if (scale_block((int)p->format) && (p->chunk_bytes % 256 || n_elems % (uint64_t)scale_block((int)p->format))) return ZCO_ERR_ARG;
    if (p->policy > 1 || p->payload_order > 1) return ZCO_ERR_ARG;
    return ZCO_OK;
}

static int limit_for(const zco_params *p, int f)
{
    int sb = zco_sym_bits((int)p->format, f);
    int L = (int)p->max_code_len[f];
    if (L == 0) L = sb == 8 ? 16 : 8;
    return L;
}

static uint64_t elems_per_chunk(const zco_params *p) { return (uint64_t)p->chunk_bytes * 8 / (uint64_t)elem_bits((int)p->format); }

/* symbols of field f inside chunk c (the last chunk may be short) */
static uint64_t chunk_symbols(const zco_params *p, int f, uint64_t n_elems, uint64_t c, uint64_t *first)
{
    uint64_t E = elems_per_chunk(p);
    uint64_t lo = c * E, hi = lo + E;
    if (hi > n_elems) hi = n_elems;
    if (f == 2) { lo /= (uint64_t)scale_block((int)p->format); hi /= (uint64_t)scale_block((int)p->format); }
    else { uint64_t g = (uint64_t)group_of((int)p->format); lo /= g; hi = (hi + g - 1) / g; }   /* E is a multiple of g */
    *first = lo;
    return hi - lo;
}

uint64_t zco_compress_bound(uint64_t n_elems, const zco_params *p)
{
    int S;
    if (check_params(p, n_elems, &S)) return 0;
    int nf = zco_num_fields((int)p->format);
    uint64_t E = elems_per_chunk(p), nc = (n_elems + E - 1) / E, total = ZCO_HEADER_BYTES;
    for (int f = 0; f < nf; f++) {
        total += pad16((uint64_t)1 << zco_sym_bits((int)p->format, f)) + pad16(4 * (nc + 1));
        total += nc * ((uint64_t)S * 12 + 32) + pad16(num_symbols((int)p->format, f, n_elems) * 2);
    }
    return total;
}

/* The coded symbols of every field of a tensor, one per byte, in freshly allocated arrays:
 * field split (+ XOR delta), then byte grouping for the formats that have it. */
static void tensor_symbols(int fmt, const uint8_t *src, const uint8_t *xor_base, const uint8_t *scales,
                           uint64_t n_elems, uint8_t *sym[3])
{
    int nf = zco_num_fields(fmt);
    uint8_t *e = malloc((size_t)n_elems + 1), *m = malloc((size_t)n_elems + 1);
    zco_split(fmt, src, xor_base, n_elems, e, m);
    sym[0] = e; sym[1] = m; sym[2] = NULL;
    if (group_of(fmt) > 1) {
        sym[0] = malloc((size_t)num_symbols(fmt, 0, n_elems) + 1); sym[1] = malloc((size_t)num_symbols(fmt, 1, n_elems) + 1);
        zco_group_values(fmt, 0, e, n_elems, sym[0]);
        zco_group_values(fmt, 1, m, n_elems, sym[1]);
        free(e); free(m);
    }
    if (nf == 3) { size_t ns = (size_t)num_symbols(fmt, 2, n_elems); sym[2] = malloc(ns + 1); if (ns) memcpy(sym[2], scales, ns); }
}

/* Compress.  src: the tensor (FP4: two elements per byte, element 2i in the low
 * nibble).  xor_base: NULL or a tensor of the same shape.  scales: FP4 only,
 * n_elems/32 E8M0 bytes.  Returns a status; *out_bytes = container size. */
static int compress_impl(const uint8_t *src, uint64_t n_elems, const zco_params *p, const uint8_t *xor_base,
                         const uint8_t *scales, const uint8_t *static_len, const uint8_t *static_mode,
                         uint8_t *dst, uint64_t cap, uint64_t *out_bytes)
{
    int S, rc = check_params(p, n_elems, &S);
    if (rc) return rc;
    int fmt = (int)p->format, nf = zco_num_fields(fmt);
    if (nf == 3 && n_elems && !scales) return ZCO_ERR_ARG;
    uint64_t E = elems_per_chunk(p), nc = (n_elems + E - 1) / E;
    if (nc > 0xFFFFFFFFu) return ZCO_ERR_ARG;

    /* 1. split into per-field symbol arrays (one symbol per byte) */
    uint8_t *sym[3] = { 0, 0, 0 };
    tensor_symbols(fmt, src, xor_base, scales, n_elems, sym);

    /* 2. histogram, mode, code per field (one code per field per tensor) */
    uint8_t len[3][256], mode[3], lmax[3], konst[3];
    uint16_t code[3][256];
    for (int f = 0; f < nf; f++) {
        uint64_t hist[256], ns = num_symbols(fmt, f, n_elems), bits = 0;
        int sb = zco_sym_bits(fmt, f), A = 1 << sb, distinct = 0;
        zco_histogram(sym[f], ns, hist);
        memset(len[f], 0, 256); memset(code[f], 0, sizeof(code[f]));
        mode[f] = ZCO_MODE_EMPTY; lmax[f] = 0; konst[f] = 0;
        for (int v = 0; v < A; v++) if (hist[v]) { distinct++; konst[f] = (uint8_t)v; }
        if (static_len && ns) {
            /* Sec. 3.3 / 5.2: a precomputed (static) dictionary is used as given, no histogram of this tensor
             * enters the code.  It must be able to code every symbol: all 2^sym_bits lengths present. */
            mode[f] = static_mode[f];
            if (mode[f] == ZCO_MODE_HUFF) {
                uint64_t kraft = 0;
                for (int v = 0; v < A; v++) {
                    len[f][v] = static_len[256 * f + v];
                    if (len[f][v] == 0 || len[f][v] > 16) { rc = ZCO_ERR_ARG; goto done; }
                    kraft += (uint64_t)1 << (16 - len[f][v]);
                    if (len[f][v] > lmax[f]) lmax[f] = len[f][v];
                }
                if (kraft != 65536) { rc = ZCO_ERR_ARG; goto done; }
                zco_canonical_codes(len[f], A, code[f]);
            } else if (mode[f] != ZCO_MODE_RAW) { rc = ZCO_ERR_ARG; goto done; }
            konst[f] = 0;
        } else if (distinct == 1) mode[f] = ZCO_MODE_CONST;
        else if (distinct > 1) {
            konst[f] = 0;
            if (zco_code_lengths(hist, A, limit_for(p, f), len[f])) { rc = ZCO_ERR_ARG; goto done; }
            for (int v = 0; v < A; v++) { bits += hist[v] * len[f][v]; if (len[f][v] > lmax[f]) lmax[f] = len[f][v]; }
            mode[f] = ZCO_MODE_HUFF;
            /* Sec. 3.1: a stream that does not compress is stored as is.  Reading:
             * under the AUTO policy Huffman must save at least 1/16 of the field. */
            if (p->policy == ZCO_POLICY_AUTO && 16 * bits > 15 * ns * (uint64_t)sb) {
                mode[f] = ZCO_MODE_RAW; memset(len[f], 0, 256); lmax[f] = 0;
            } else zco_canonical_codes(len[f], A, code[f]);
        }
    }

    /* 3. layout */
    uint64_t off = ZCO_HEADER_BYTES, table_off[3], index_off[3];
    for (int f = 0; f < nf; f++) { table_off[f] = off; off += pad16((uint64_t)1 << zco_sym_bits(fmt, f)); }
    for (int f = 0; f < nf; f++) { index_off[f] = off; off += pad16(4 * (nc + 1)); }
    uint64_t payload_off = off;
    if (payload_off > cap) { rc = ZCO_ERR_SMALL; goto done; }
    memset(dst, 0, (size_t)payload_off);

    /* 4. streams, field-major, the fields in the payload's order */
    uint64_t units = 0;                                   /* payload size so far, 16-byte units */
    for (int k = 0; k < nf; k++) {
        int f = p->payload_order ? nf - 1 - k : k;
        int sb = zco_sym_bits(fmt, f), G = run_len(fmt, f);
        for (uint64_t c = 0; c < nc; c++) {
            uint64_t first, n = chunk_symbols(p, f, n_elems, c, &first), bytes = 0;
            put32(dst + index_off[f] + 4 * c, (uint32_t)units);
            if (mode[f] == ZCO_MODE_HUFF) {
                if (payload_off + 16 * units + zco_stream_bound(n, S, lmax[f]) > cap) { rc = ZCO_ERR_SMALL; goto done; }
                bytes = zco_encode_stream(sym[f] + first, n, len[f], code[f], lmax[f], G, S, dst + payload_off + 16 * units);
            } else if (mode[f] == ZCO_MODE_RAW) {
                if (payload_off + 16 * units + raw_stream_bytes(n, sb) > cap) { rc = ZCO_ERR_SMALL; goto done; }
                bytes = encode_raw(sym[f] + first, n, sb, dst + payload_off + 16 * units);
            }
            units += bytes / 16;
            if (units > 0xFFFFFFFFu) { rc = ZCO_ERR_ARG; goto done; }
        }
        put32(dst + index_off[f] + 4 * nc, (uint32_t)units);
    }
    uint64_t total = payload_off + 16 * units;

    /* 5. header and tables */
    put32(dst + 0, ZCO_MAGIC);
    dst[4] = 1; dst[5] = 0; dst[6] = (uint8_t)fmt; dst[7] = (uint8_t)p->policy;
    dst[8] = (uint8_t)S; dst[9] = (uint8_t)nf; dst[10] = (uint8_t)((xor_base ? 1 : 0) | (p->payload_order ? 2 : 0));
    put32(dst + 12, p->chunk_bytes);
    put64(dst + 16, n_elems);
    put32(dst + 24, (uint32_t)nc);
    for (int f = 0; f < nf; f++) {
        dst[32 + 4 * f + 0] = mode[f]; dst[32 + 4 * f + 1] = (uint8_t)zco_sym_bits(fmt, f);
        dst[32 + 4 * f + 2] = lmax[f]; dst[32 + 4 * f + 3] = konst[f];
        memcpy(dst + table_off[f], len[f], (size_t)1 << zco_sym_bits(fmt, f));
    }
    put64(dst + 48, total);
    put64(dst + 56, payload_off);
    *out_bytes = total;
done:
    free(sym[0]); free(sym[1]); free(sym[2]);
    return rc;
}

int zco_compress(const uint8_t *src, uint64_t n_elems, const zco_params *p, const uint8_t *xor_base,
                 const uint8_t *scales, uint8_t *dst, uint64_t cap, uint64_t *out_bytes)
{
    return compress_impl(src, n_elems, p, xor_base, scales, NULL, NULL, dst, cap, out_bytes);
}

/* Compress with a code computed ahead of time on other, representative data (Sec. 3.3 and 5.2:
 * static dictionaries for K/V caches whose exponent distribution stays stable).
 * static_len: 3 x 256 code lengths, static_mode: 3 modes (HUFF or RAW). */
int zco_compress_with_code(const uint8_t *src, uint64_t n_elems, const zco_params *p, const uint8_t *xor_base,
                           const uint8_t *scales, const uint8_t *static_len, const uint8_t *static_mode,
                           uint8_t *dst, uint64_t cap, uint64_t *out_bytes)
{
    if (!static_len || !static_mode) return ZCO_ERR_ARG;
    return compress_impl(src, n_elems, p, xor_base, scales, static_len, static_mode, dst, cap, out_bytes);
}

/* Train a static dictionary on representative data: the tensor's histogram with every count
 * raised by one (so that every symbol of the alphabet can be coded later), then the same code
 * construction and the same raw/Huffman decision as zco_compress. */
int zco_train_code(const uint8_t *src, uint64_t n_elems, const zco_params *p, const uint8_t *xor_base,
                   const uint8_t *scales, uint8_t *len_out /* 3 x 256 */, uint8_t *mode_out /* 3 */)
{
    int S, rc = check_params(p, n_elems, &S);
    if (rc) return rc;
    int fmt = (int)p->format, nf = zco_num_fields(fmt);
    uint8_t *sym[3];
    if (nf == 3 && n_elems && !scales) return ZCO_ERR_ARG;
    tensor_symbols(fmt, src, xor_base, scales, n_elems, sym);
    memset(len_out, 0, 768); memset(mode_out, 0, 3);
    for (int f = 0; f < nf && !rc; f++) {
        const uint8_t *syms = sym[f];
        uint64_t hist[256], ns = num_symbols(fmt, f, n_elems), bits = 0, total = 0;
        int sb = zco_sym_bits(fmt, f), A = 1 << sb;
        zco_histogram(syms, ns, hist);
        for (int v = 0; v < A; v++) { hist[v] += 1; total += hist[v]; }
        if (zco_code_lengths(hist, A, limit_for(p, f), len_out + 256 * f)) { rc = ZCO_ERR_ARG; break; }
        for (int v = 0; v < A; v++) bits += hist[v] * len_out[256 * f + v];
        mode_out[f] = ZCO_MODE_HUFF;
        if (p->policy == ZCO_POLICY_AUTO && 16 * bits > 15 * total * (uint64_t)sb) { mode_out[f] = ZCO_MODE_RAW; memset(len_out + 256 * f, 0, 256); }
    }
    free(sym[0]); free(sym[1]); free(sym[2]);
    return rc;
}

/* parsed view of a container */
typedef struct {
    int fmt, policy, S, nf, xor_flag, reversed;
    uint32_t chunk_bytes;
    uint64_t n_elems, nc, total, payload_off, table_off[3], index_off[3];
    uint8_t mode[3], sym_bits[3], lmax[3], konst[3];
} zco_view;

static int parse(const uint8_t *c, uint64_t bytes, zco_view *v)
{
    if (bytes < ZCO_HEADER_BYTES || get32(c) != ZCO_MAGIC || c[4] != 1 || c[5] != 0) return ZCO_ERR_CORRUPT;
    v->fmt = c[6]; v->policy = c[7]; v->S = c[8]; v->nf = c[9]; v->xor_flag = c[10] & 1; v->reversed = (c[10] >> 1) & 1;
    v->chunk_bytes = get32(c + 12); v->n_elems = get64(c + 16); v->nc = get32(c + 24);
    v->total = get64(c + 48); v->payload_off = get64(c + 56);
    zco_params p; memset(&p, 0, sizeof(p));
    p.format = (uint32_t)v->fmt; p.chunk_bytes = v->chunk_bytes; p.streams_per_chunk = (uint32_t)v->S; p.policy = (uint32_t)v->policy;
    int S;
    if (!elem_bits(v->fmt) || v->S == 0 || check_params(&p, v->n_elems, &S) || v->nf != zco_num_fields(v->fmt)) return ZCO_ERR_CORRUPT;
    uint64_t E = elems_per_chunk(&p);
    if (v->nc != (v->n_elems + E - 1) / E || v->total > bytes) return ZCO_ERR_CORRUPT;
    uint64_t off = ZCO_HEADER_BYTES;
    for (int f = 0; f < v->nf; f++) {
        v->mode[f] = c[32 + 4 * f]; v->sym_bits[f] = c[32 + 4 * f + 1]; v->lmax[f] = c[32 + 4 * f + 2]; v->konst[f] = c[32 + 4 * f + 3];
        if (v->mode[f] > 3 || v->sym_bits[f] != zco_sym_bits(v->fmt, f)) return ZCO_ERR_CORRUPT;
        v->table_off[f] = off; off += pad16((uint64_t)1 << v->sym_bits[f]);
    }
    for (int f = 0; f < v->nf; f++) { v->index_off[f] = off; off += pad16(4 * (v->nc + 1)); }
    if (off != v->payload_off || off > v->total) return ZCO_ERR_CORRUPT;
    /* chunk offsets must not decrease and must end inside the container */
    uint32_t prev = 0;
    for (int k = 0; k < v->nf; k++)
        for (uint64_t i = 0; i <= v->nc; i++) {
            int f = v->reversed ? v->nf - 1 - k : k;
            uint32_t o = get32(c + v->index_off[f] + 4 * i);
            if (o < prev || (i == 0 && o != prev)) return ZCO_ERR_CORRUPT;
            prev = o;
        }
    if (v->payload_off + 16 * (uint64_t)prev != v->total) return ZCO_ERR_CORRUPT;
    return ZCO_OK;
}

/* decode the symbols of field f of chunk c into out (one symbol per byte) */
static int decode_field_chunk(const uint8_t *comp, const zco_view *v, int f, uint64_t c, uint64_t n, uint8_t *out)
{
    uint64_t a = get32(comp + v->index_off[f] + 4 * c), b = get32(comp + v->index_off[f] + 4 * (c + 1));
    const uint8_t *in = comp + v->payload_off + 16 * a;
    uint64_t avail = 16 * (b - a);
    if (v->mode[f] == ZCO_MODE_CONST) { memset(out, v->konst[f], (size_t)n); return avail ? ZCO_ERR_CORRUPT : ZCO_OK; }
    if (v->mode[f] == ZCO_MODE_EMPTY) return (n || avail) ? ZCO_ERR_CORRUPT : ZCO_OK;
    if (v->mode[f] == ZCO_MODE_RAW) {
        if (avail != raw_stream_bytes(n, v->sym_bits[f])) return ZCO_ERR_CORRUPT;
        decode_raw(in, n, v->sym_bits[f], out);
        return ZCO_OK;
    }
    uint64_t used = zco_decode_stream(in, avail, n, comp + v->table_off[f], 1 << v->sym_bits[f],
                                      run_len(v->fmt, f), v->S, out);
    if (n == 0) return avail ? ZCO_ERR_CORRUPT : ZCO_OK;
    return used == avail ? ZCO_OK : ZCO_ERR_CORRUPT;
}

/* Decode chunk c alone: dst gets the chunk's element bytes, scales_out (FP4)
 * its scale bytes; xor_base_chunk is the matching slice of the base tensor. */
int zco_decompress_chunk(const uint8_t *comp, uint64_t comp_bytes, uint64_t c, const uint8_t *xor_base_chunk,
                         uint8_t *dst, uint64_t dst_cap, uint8_t *scales_out)
{
    zco_view v;
    int rc = parse(comp, comp_bytes, &v);
    if (rc) return rc;
    if (c >= v.nc) return ZCO_ERR_ARG;
    if (v.xor_flag && !xor_base_chunk) return ZCO_ERR_ARG;
    zco_params p; memset(&p, 0, sizeof(p));
    p.format = (uint32_t)v.fmt; p.chunk_bytes = v.chunk_bytes;
    uint64_t first, ns01 = chunk_symbols(&p, 0, v.n_elems, c, &first);
    uint64_t E = elems_per_chunk(&p), n = v.n_elems - c * E < E ? v.n_elems - c * E : E;    /* elements in the chunk */
    uint64_t out_bytes = (n * (uint64_t)elem_bits(v.fmt) + 7) / 8;
    if (out_bytes > dst_cap) return ZCO_ERR_SMALL;
    uint8_t *e = malloc((size_t)n + 1), *m = malloc((size_t)n + 1);
    if (group_of(v.fmt) == 1) {
        rc = decode_field_chunk(comp, &v, 0, c, n, e);
        if (!rc) rc = decode_field_chunk(comp, &v, 1, c, n, m);
    } else {
        uint8_t *s0 = malloc((size_t)ns01 + 1), *s1 = malloc((size_t)ns01 + 1);
        rc = decode_field_chunk(comp, &v, 0, c, ns01, s0);
        if (!rc) rc = decode_field_chunk(comp, &v, 1, c, ns01, s1);
        if (!rc) { zco_ungroup_symbols(v.fmt, 0, s0, n, e); zco_ungroup_symbols(v.fmt, 1, s1, n, m); }
        free(s0); free(s1);
    }
    if (!rc) zco_join(v.fmt, e, m, v.xor_flag ? xor_base_chunk : NULL, n, dst);
    if (!rc && v.nf == 3) {
        uint64_t ns = chunk_symbols(&p, 2, v.n_elems, c, &first);
        if (!scales_out) rc = ZCO_ERR_ARG; else rc = decode_field_chunk(comp, &v, 2, c, ns, scales_out);
    }
    free(e); free(m);
    return rc;
}

int zco_decompress(const uint8_t *comp, uint64_t comp_bytes, const uint8_t *xor_base,
                   uint8_t *dst, uint64_t dst_cap, uint8_t *scales_out)
{
    zco_view v;
    int rc = parse(comp, comp_bytes, &v);
    if (rc) return rc;
    if ((v.n_elems * (uint64_t)elem_bits(v.fmt) + 7) / 8 > dst_cap) return ZCO_ERR_SMALL;
    if (v.xor_flag && !xor_base && v.n_elems) return ZCO_ERR_ARG;
    for (uint64_t c = 0; c < v.nc && !rc; c++) {
        uint64_t eoff = c * (uint64_t)v.chunk_bytes;
        rc = zco_decompress_chunk(comp, comp_bytes, c, xor_base ? xor_base + eoff : NULL, dst + eoff,
                                  dst_cap - eoff, scales_out ? scales_out + c * ((uint64_t)v.chunk_bytes * 2 / (uint64_t)scale_block(v.fmt)) : NULL);
    }
    return rc;
}

/* ------------------------------------------------------------------- stats */
/* Sec. 4: compression ratio and its per-component breakdown.  ratio = coded
 * size / original size (lower is better), as the paper uses the word. */
typedef struct {
    uint32_t alphabet, distinct, mode, max_len;
    uint64_t n_symbols;
    uint64_t hist[256];
    uint8_t code_len[256];
    double entropy_bits;       /* H = -sum p log2 p, bits per symbol */
    double mean_code_len;      /* sum f*len / n */
    uint64_t payload_bits;     /* sum f*len (HUFF), n*sym_bits (RAW), 0 (CONST) */
    uint64_t stream_bytes;     /* bytes of this field's streams in the container */
    double ratio_payload;      /* payload_bits / (n*sym_bits) */
} zco_field_stats;

typedef struct {
    uint32_t n_fields, pad;
    uint64_t raw_bytes;        /* element bytes + scale bytes */
    uint64_t container_bytes;
    double ratio_payload_total;    /* sum payload_bits / (8*raw_bytes) */
    double ratio_container_total;  /* container_bytes / raw_bytes */
    zco_field_stats field[3];
} zco_stats_out;

int zco_stats(const uint8_t *src, uint64_t n_elems, const zco_params *p, const uint8_t *xor_base,
              const uint8_t *scales, zco_stats_out *out)
{
    int S, rc = check_params(p, n_elems, &S);
    if (rc) return rc;
    int fmt = (int)p->format, nf = zco_num_fields(fmt);
    memset(out, 0, sizeof(*out));
    out->n_fields = (uint32_t)nf;
    out->raw_bytes = (n_elems * (uint64_t)elem_bits(fmt) + 7) / 8 + (nf == 3 ? num_symbols(fmt, 2, n_elems) : 0);
    uint64_t cap = zco_compress_bound(n_elems, p), total = 0;
    uint8_t *tmp = malloc((size_t)cap);
    rc = zco_compress(src, n_elems, p, xor_base, scales, tmp, cap, &total);
    if (rc) { free(tmp); return rc; }
    zco_view v;
    parse(tmp, total, &v);
    out->container_bytes = total;
    uint8_t *sym[3];
    tensor_symbols(fmt, src, xor_base, scales, n_elems, sym);
    uint64_t all_bits = 0;
    for (int f = 0; f < nf; f++) {
        zco_field_stats *fs = &out->field[f];
        const uint8_t *syms = sym[f];
        int sb = zco_sym_bits(fmt, f);
        fs->alphabet = 1u << sb; fs->n_symbols = num_symbols(fmt, f, n_elems); fs->mode = v.mode[f]; fs->max_len = v.lmax[f];
        zco_histogram(syms, fs->n_symbols, fs->hist);
        memcpy(fs->code_len, tmp + v.table_off[f], (size_t)1 << sb);
        for (unsigned s = 0; s < fs->alphabet; s++) if (fs->hist[s]) {
            double pr = (double)fs->hist[s] / (double)fs->n_symbols;
            fs->distinct++;
            fs->entropy_bits -= pr * log2(pr);
            if (fs->mode == ZCO_MODE_HUFF) fs->payload_bits += fs->hist[s] * fs->code_len[s];
        }
        if (fs->mode == ZCO_MODE_RAW) fs->payload_bits = fs->n_symbols * (uint64_t)sb;
        if (fs->n_symbols) {
            fs->mean_code_len = (double)fs->payload_bits / (double)fs->n_symbols;
            fs->ratio_payload = (double)fs->payload_bits / ((double)fs->n_symbols * sb);
        }
        fs->stream_bytes = 16 * ((uint64_t)get32(tmp + v.index_off[f] + 4 * v.nc) - (uint64_t)get32(tmp + v.index_off[f]));
        all_bits += fs->payload_bits;
    }
    if (out->raw_bytes) {
        out->ratio_payload_total = (double)all_bits / (8.0 * (double)out->raw_bytes);
        out->ratio_container_total = (double)total / (double)out->raw_bytes;
    }
    free(sym[0]); free(sym[1]); free(sym[2]); free(tmp);
    return ZCO_OK;
}
