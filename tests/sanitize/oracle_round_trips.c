/* Random round trips of every format through the oracle, meant to be built with -fsanitize=address,undefined
 * (tests/test_sanitizers.py): the decompressor gets a heap copy of exactly the container's bytes, so a read
 * past its end is caught. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
typedef struct { uint32_t format, chunk_bytes, max_code_len[3], streams_per_chunk, policy, payload_order; } zco_params;
int zco_compress(const uint8_t *src, uint64_t n_elems, const zco_params *p, const uint8_t *xor_base, const uint8_t *scales, uint8_t *dst, uint64_t cap, uint64_t *out_bytes);
int zco_decompress(const uint8_t *comp, uint64_t comp_bytes, const uint8_t *xor_base, uint8_t *dst, uint64_t dst_cap, uint8_t *scales_out);
uint64_t zco_compress_bound(uint64_t n_elems, const zco_params *p);
static uint64_t s = 88172645463325252ull;
static uint64_t rnd(void) { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; }
int main(void) {
    const int ebits[8] = {0, 16, 8, 4, 8, 4, 4, 8};
    const int sblock[8] = {0, 0, 0, 32, 0, 32, 16, 0};
    long done = 0;
    for (int it = 0; it < 1200; it++) {
        int fmt = 1 + rnd() % 7;
        int unit = sblock[fmt] ? 256 : 16;
        zco_params p; memset(&p, 0, sizeof p);
        p.format = fmt; p.chunk_bytes = unit * (1 + rnd() % 20); p.streams_per_chunk = 1u << (rnd() % 7); p.policy = rnd() % 2; p.payload_order = rnd() % 2;
        uint64_t E = (uint64_t)p.chunk_bytes * 8 / ebits[fmt];
        uint64_t n = rnd() % (4 * E + 2);
        if (sblock[fmt]) n = n / sblock[fmt] * sblock[fmt];
        uint64_t bytes = (n * ebits[fmt] + 7) / 8, nsc = sblock[fmt] ? n / sblock[fmt] : 0;
        uint8_t *src = malloc(bytes + 1), *base = malloc(bytes + 1), *sc = malloc(nsc + 1), *out = malloc(bytes + 1), *sco = malloc(nsc + 1);
        int skew = rnd() % 3;
        for (uint64_t i = 0; i < bytes; i++) { src[i] = skew == 0 ? rnd() : skew == 1 ? (rnd() % 7) * 9 : ((rnd() % 16 ? 0x38 : rnd()) & 0xFF); base[i] = rnd() & 0x81; }
        for (uint64_t i = 0; i < nsc; i++) sc[i] = 118 + rnd() % 5;
        int delta = rnd() % 3 == 0;
        uint64_t cap = zco_compress_bound(n, &p), got = 0;
        if (cap == 0) { printf("bound 0 fmt %d\n", fmt); return 1; }
        uint8_t *comp = malloc(cap);
        int rc = zco_compress(src, n, &p, delta ? base : NULL, nsc ? sc : NULL, comp, cap, &got);
        if (rc) { printf("compress rc %d fmt %d n %llu\n", rc, fmt, (unsigned long long)n); return 1; }
        uint8_t *exact = malloc(got ? got : 1); memcpy(exact, comp, got);     /* so that reads past the container are caught */
        rc = zco_decompress(exact, got, delta ? base : NULL, out, bytes, nsc ? sco : NULL);
        if (rc || memcmp(out, src, bytes) || (nsc && memcmp(sco, sc, nsc))) { printf("round trip failed rc %d fmt %d n %llu\n", rc, fmt, (unsigned long long)n); return 1; }
        free(src); free(base); free(sc); free(out); free(sco); free(comp); free(exact);
        done++;
    }
    printf("ok %ld\n", done);
    return 0;
}
