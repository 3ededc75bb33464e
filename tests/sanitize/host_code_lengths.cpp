// Random histograms through the library's host-side code construction, meant to be built with
// -fsanitize=address,undefined (tests/test_sanitizers.py); checks that every code is complete.
#include "zc_internal.h"
#include <cstdio>
#include <cstdlib>
#include <random>
using namespace zc;
int main() {
    std::mt19937_64 rng(7);
    long checked = 0;
    for (int it = 0; it < 8000; it++) {
        int A = 1 << (1 + rng() % 8);
        uint64_t h[256] = {0};
        int kind = rng() % 5;
        for (int v = 0; v < A; v++) {
            if (kind == 0) h[v] = rng() % 3 ? rng() % 1000 : 0;
            else if (kind == 1) h[v] = (rng() % 4) ? 0 : (1ull << (rng() % 40));
            else if (kind == 2) h[v] = 1;
            else if (kind == 3) h[v] = rng() % 2 ? (uint64_t)(rng() >> (rng() % 60)) >> 8 : 0;
            else h[v] = v < 40 ? (1ull << (v % 45)) : 0;
        }
        int limit = 1 + rng() % 16;
        uint8_t len[256]; uint16_t code[256];
        if (!build_code_lengths(h, A, limit, len)) continue;
        assign_canonical(len, A, code);
        unsigned long long kraft = 0; int n = 0;
        for (int v = 0; v < A; v++) if (len[v]) { if (len[v] > 16) { printf("len>16\n"); return 1; } kraft += 1ull << (16 - len[v]); n++; }
        if (n >= 2 && kraft != 65536) { printf("kraft %llu n %d limit %d\n", kraft, n, limit); return 1; }
        checked++;
    }
    printf("ok %ld\n", checked);
    return 0;
}
