// Host-side Huffman code construction for the two entry arrays (value indices and
// relative indices, Sec. III-B last paragraph).  Codes are length-limited so that a
// flat decode table indexed by CL_MAX_CODE_LEN stream bits fits in LDS, and
// canonical so that only the lengths need storing.
#include <algorithm>
#include <functional>
#include <queue>

#include "layer.hpp"

namespace cl {

namespace {
struct Item {
    uint64_t weight;
    std::vector<uint16_t> uses;   // how many times each used symbol occurs inside this package
};
}  // namespace

bool limited_code_lengths(const std::vector<int64_t> &counts, int limit, std::vector<uint8_t> &len)
{
    const int nsym = (int)counts.size();
    len.assign(nsym, 0);
    std::vector<int> used;
    for (int s = 0; s < nsym; ++s)
        if (counts[s] > 0) used.push_back(s);
    const int n = (int)used.size();
    if (n == 0) return true;
    if (n == 1) { len[used[0]] = 1; return true; }
    if (limit < 1 || limit > 31 || (1ll << limit) < n) return false;
    std::stable_sort(used.begin(), used.end(), [&](int a, int b) { return counts[a] < counts[b]; });

    // Package-merge: at each of `limit` levels the list is the sorted leaves merged
    // with pairs ("packages") of the previous level's list.  The 2n - 2 cheapest
    // items of the last list cover every leaf once per bit of its codeword.
    std::vector<Item> leaves(n);
    for (int i = 0; i < n; ++i) {
        leaves[i].weight = (uint64_t)counts[used[i]];
        leaves[i].uses.assign(n, 0);
        leaves[i].uses[i] = 1;
    }
    std::vector<Item> prev = leaves, cur;
    for (int level = 2; level <= limit; ++level) {
        std::vector<Item> packs;
        for (size_t i = 0; i + 1 < prev.size(); i += 2) {
            Item p;
            p.weight = prev[i].weight + prev[i + 1].weight;
            p.uses = prev[i].uses;
            for (int j = 0; j < n; ++j) p.uses[j] = (uint16_t)(p.uses[j] + prev[i + 1].uses[j]);
            packs.push_back(std::move(p));
        }
        cur.clear();
        cur.reserve(leaves.size() + packs.size());
        size_t a = 0, b = 0;
        while (a < leaves.size() || b < packs.size()) {
            if (b >= packs.size() || (a < leaves.size() && leaves[a].weight <= packs[b].weight)) cur.push_back(leaves[a++]);
            else cur.push_back(std::move(packs[b++]));
        }
        prev.swap(cur);
    }
    std::vector<int> l(n, 0);
    const size_t take = (size_t)(2 * n - 2);
    for (size_t i = 0; i < take && i < prev.size(); ++i)
        for (int j = 0; j < n; ++j) l[j] += prev[i].uses[j];
    for (int i = 0; i < n; ++i) len[used[i]] = (uint8_t)l[i];
    return true;
}

int64_t unlimited_code_bits(const std::vector<int64_t> &counts)
{
    std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> pq;
    for (int64_t c : counts)
        if (c > 0) pq.push(c);
    if (pq.empty()) return 0;
    if (pq.size() == 1) return pq.top();
    int64_t bits = 0;
    while (pq.size() > 1) {
        int64_t a = pq.top(); pq.pop();
        int64_t b = pq.top(); pq.pop();
        bits += a + b;
        pq.push(a + b);
    }
    return bits;
}

bool canonical_codes(const std::vector<uint8_t> &len, std::vector<uint32_t> &code, int *max_len)
{
    const int nsym = (int)len.size();
    code.assign(nsym, 0);
    int mx = 0;
    for (int s = 0; s < nsym; ++s) mx = std::max<int>(mx, len[s]);
    *max_len = mx;
    if (mx == 0) return true;
    if (mx > CL_MAX_CODE_LEN) return false;
    // Kraft: sum 2^(mx - len) <= 2^mx
    uint64_t kraft = 0;
    for (int s = 0; s < nsym; ++s)
        if (len[s]) kraft += 1ull << (mx - len[s]);
    if (kraft > (1ull << mx)) return false;
    // shorter codewords first, then by symbol; numeric value counts up
    uint32_t next = 0;
    int prev_len = 0;
    for (int l = 1; l <= mx; ++l)
        for (int s = 0; s < nsym; ++s) {
            if (len[s] != l) continue;
            next <<= (l - prev_len);
            prev_len = l;
            // the codeword's most significant bit is written to the stream first
            uint32_t rev = 0;
            for (int j = 0; j < l; ++j) rev |= ((next >> (l - 1 - j)) & 1u) << j;
            code[s] = rev;
            ++next;
        }
    return true;
}

void build_lut(const std::vector<uint8_t> &len, const std::vector<uint32_t> &code, int max_len,
               std::vector<lut_t> &lut)
{
    const int bits = std::max(1, max_len);
    // Slots no codeword reaches (incomplete codes) still advance by one bit, so a
    // decoder loop always terminates.
    lut.assign((size_t)1 << bits, (lut_t)1u);
    for (int s = 0; s < (int)len.size(); ++s) {
        const int l = len[s];
        if (!l) continue;
        for (uint32_t hi = 0; hi < (1u << (bits - l)); ++hi)
            lut[(hi << l) | code[s]] = (lut_t)((s << 8) | l);
    }
}

}  // namespace cl
