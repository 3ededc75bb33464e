// Host-side Huffman code construction for alphabets of at most 256 symbols:
// optimal code lengths under a length limit (package-merge, Larmore & Hirschberg 1990),
// then canonical code values.  The paper asks only for plain Huffman coding per stream
// (Sec. 3.1, 4.1); the limit keeps decode tables small and the tie rules below make the
// result unique so that an independent implementation arrives at the same bits:
//   * leaves are ordered by (frequency, symbol value), ascending;
//   * when a row is merged, a leaf goes before a package of equal weight;
//   * canonical codes are handed out in (length, symbol value) order.
//
// This implementation keeps only weights and leaf flags per row and recovers the lengths
// by walking down the rows with a running item budget (the "boundary" form), so a row
// never stores which leaves a package contains.
#include "zc_internal.h"

#include <algorithm>
#include <cstring>
#include <vector>

namespace zc {

bool build_code_lengths(const uint64_t *hist, int alphabet, int limit, uint8_t *len_out)
{
    std::memset(len_out, 0, (size_t)alphabet);
    std::vector<int> order;
    for (int v = 0; v < alphabet; v++)
        if (hist[v]) order.push_back(v);
    const int n = (int)order.size();
    if (n == 0) return true;
    if (n == 1) { len_out[order[0]] = 1; return true; }
    if (limit < 1 || limit > 16 || (1 << limit) < n) return false;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return hist[a] < hist[b]; });

    struct Row { std::vector<uint64_t> w; std::vector<uint8_t> leaf; };
    std::vector<Row> rows((size_t)limit + 1);          // rows[1..limit]; rows[limit] holds the leaves only
    Row &bottom = rows[(size_t)limit];
    for (int i = 0; i < n; i++) { bottom.w.push_back(hist[order[i]]); bottom.leaf.push_back(1); }
    for (int d = limit - 1; d >= 1; d--) {
        const Row &below = rows[(size_t)d + 1];
        Row &cur = rows[(size_t)d];
        const size_t n_pk = below.w.size() / 2;
        size_t a = 0, b = 0;
        cur.w.reserve((size_t)n + n_pk);
        cur.leaf.reserve((size_t)n + n_pk);
        while (a < (size_t)n || b < n_pk) {
            const uint64_t pw = b < n_pk ? below.w[2 * b] + below.w[2 * b + 1] : 0;
            if (b >= n_pk || (a < (size_t)n && hist[order[a]] <= pw)) { cur.w.push_back(hist[order[a]]); cur.leaf.push_back(1); a++; }
            else { cur.w.push_back(pw); cur.leaf.push_back(0); b++; }
        }
    }
    // Take the cheapest 2n-2 items of the top row; every package taken there stands for two
    // items of the row below, and so on.  The i-th cheapest leaf is used once per row in
    // which it lies inside the budget, and that count is its code length.
    size_t budget = 2 * (size_t)n - 2;
    for (int d = 1; d <= limit && budget > 0; d++) {
        const Row &row = rows[(size_t)d];
        if (budget > row.w.size()) budget = row.w.size();
        size_t leaves = 0;
        for (size_t i = 0; i < budget; i++) leaves += row.leaf[i];
        for (size_t i = 0; i < leaves; i++) len_out[order[i]]++;
        budget = 2 * (budget - leaves);
    }
    return true;
}

void assign_canonical(const uint8_t *len, int alphabet, uint16_t *code_out)
{
    // count codes per length, derive the first code of each length, then number the
    // symbols of equal length in ascending symbol order
    unsigned count[17] = {0}, next[17] = {0};
    for (int v = 0; v < alphabet; v++) count[len[v]]++;
    count[0] = 0;
    unsigned code = 0;
    for (int l = 1; l <= 16; l++) {
        code = (code + count[l - 1]) << 1;
        next[l] = code;
    }
    for (int v = 0; v < alphabet; v++) code_out[v] = len[v] ? (uint16_t)next[len[v]]++ : 0;
}

}  // namespace zc
