// The library's host-side container validation (zc_validate_container) on damaged containers, meant to be built
// with -fsanitize=address,undefined (tests/test_sanitizers.py).  Containers come from the oracle; the validator
// gets a heap copy of exactly the bytes it is told about, so a read past them is caught.  An undamaged container
// must validate; a damaged one may give any status but must not read outside the copy.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "zc.h"

extern "C" {
typedef struct { uint32_t format, chunk_bytes, max_code_len[3], streams_per_chunk, policy, payload_order; } zco_params;
int zco_compress(const uint8_t *src, uint64_t n_elems, const zco_params *p, const uint8_t *xor_base, const uint8_t *scales, uint8_t *dst, uint64_t cap, uint64_t *out_bytes);
uint64_t zco_compress_bound(uint64_t n_elems, const zco_params *p);
}

int main()
{
    std::mt19937_64 rng(11);
    long checked = 0, rejected = 0;
    for (int it = 0; it < 60; it++) {
        zco_params p;
        std::memset(&p, 0, sizeof p);
        p.format = 1 + it % 3;                                   // BF16, FP8 E4M3, MXFP4
        p.chunk_bytes = p.format == 3 ? 1024 : 2048;
        p.streams_per_chunk = 1u << (rng() % 7);
        p.policy = rng() % 2;
        p.payload_order = rng() % 2;
        const uint64_t n = p.format == 3 ? 32 * (1 + rng() % 400) : 1 + rng() % 20000;
        const uint64_t bytes = p.format == 1 ? 2 * n : p.format == 2 ? n : n / 2;
        std::vector<uint8_t> src(bytes), sc(n / 32 + 1);
        for (auto &b : src) b = (uint8_t)((rng() % 7 == 0) ? rng() : 0x3C + rng() % 3);
        for (auto &b : sc) b = (uint8_t)(120 + rng() % 4);
        const uint64_t cap = zco_compress_bound(n, &p);
        std::vector<uint8_t> comp(cap);
        uint64_t got = 0;
        if (zco_compress(src.data(), n, &p, nullptr, p.format == 3 ? sc.data() : nullptr, comp.data(), cap, &got)) { std::printf("oracle failed\n"); return 1; }
        zc_info info;
        {
            uint8_t *exact = (uint8_t *)std::malloc(got);
            std::memcpy(exact, comp.data(), got);
            const zc_status st = zc_validate_container(exact, got, got, 1, &info);
            std::free(exact);
            if (st != ZC_OK || info.total_bytes != got || info.n_elems != n) { std::printf("good container refused: %d\n", (int)st); return 1; }
        }
        for (int k = 0; k < 300; k++) {
            const uint64_t have = (k % 5 == 0) ? 1 + rng() % got : got;           // sometimes only a prefix is there
            uint8_t *exact = (uint8_t *)std::malloc(have);
            std::memcpy(exact, comp.data(), have);
            const uint64_t span = info.payload_offset < have ? info.payload_offset : have;
            const int hits = 1 + (int)(rng() % 3);
            for (int h = 0; h < hits; h++) exact[rng() % span] = (uint8_t)rng();
            zc_info out;
            const zc_status st = zc_validate_container(exact, have, (k % 7 == 0) ? have : got, (int)(rng() % 2), &out);
            rejected += st != ZC_OK;
            checked++;
            std::free(exact);
        }
    }
    std::printf("ok %ld damaged containers, %ld rejected\n", checked, rejected);
    return 0;
}
