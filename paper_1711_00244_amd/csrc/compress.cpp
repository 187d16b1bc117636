// Host side of the library: builds the compressed form of a pruned weight matrix
// (Sec. III-B pipeline, block-contiguous as in Sec. IV-A), validates it, and
// converts it to and from a relocatable byte image.  No HIP calls here.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>
#include <memory>
#include <new>

#include "layer.hpp"

namespace cl {

static thread_local std::string g_error;

int32_t fail(int32_t code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_error = buf;
    return code;
}

void clear_error() { g_error.clear(); }

namespace {

struct Geometry {
    int M, K, bh, bw;
    int nbh, nbw;
    int64_t n_blocks;
    explicit Geometry(const cl_layer_desc &d)
        : M(d.M), K(d.K), bh(d.block_h), bw(d.block_w), nbh((d.M + d.block_h - 1) / d.block_h),
          nbw((d.K + d.block_w - 1) / d.block_w), n_blocks((int64_t)nbh * nbw) {}
    // Algorithm 2: block i starts at row (i / nbw) * bh and column (i % nbw) * bw.
    void block(int64_t i, int &row_id, int &col_id, int &bhp, int &bwp) const
    {
        row_id = (int)(i / nbw) * bh;
        col_id = (int)(i % nbw) * bw;
        bhp = std::min(bh, M - row_id);
        bwp = std::min(bw, K - col_id);
    }
};

int32_t check_desc(cl_layer_desc &d)
{
    if (d.M < 1 || d.K < 1) return fail(CL_EINVAL, "M and K must be positive (got %d x %d)", d.M, d.K);
    if ((int64_t)d.M * d.K > std::numeric_limits<int32_t>::max()) return fail(CL_EINVAL, "M*K exceeds 2^31-1");
    if (d.weight_bits < 1 || d.weight_bits > 8) return fail(CL_EINVAL, "weight_bits must be in 1..8 (got %d)", d.weight_bits);
    if (d.index_bits < 1 || d.index_bits > 8) return fail(CL_EINVAL, "index_bits must be in 1..8 (got %d)", d.index_bits);
    if (d.block_h < 1 || d.block_w < 1) return fail(CL_EINVAL, "block_h and block_w must be positive");
    if (d.block_h > d.M) d.block_h = d.M;
    if (d.block_w > d.K) d.block_w = d.K;
    if (d.chunk_bits == 0) d.chunk_bits = CL_CHUNK_BITS;
    if (d.chunk_bits != CL_CHUNK_BITS) return fail(CL_EINVAL, "chunk_bits must be %d", CL_CHUNK_BITS);
    if (d.max_code_len == 0) d.max_code_len = CL_MAX_CODE_LEN;
    if (d.max_code_len > CL_MAX_CODE_LEN || d.max_code_len < std::max(d.weight_bits, d.index_bits))
        return fail(CL_EINVAL, "max_code_len must be in max(weight_bits,index_bits)..%d", CL_MAX_CODE_LEN);
    return CL_OK;
}

inline uint64_t bit_reverse64(uint64_t x)
{
    uint64_t r = 0;
    for (int i = 0; i < 64; ++i) r |= ((x >> i) & 1ull) << (63 - i);
    return r;
}

}  // namespace

// --------------------------------------------------------------------------- //
// Everything that can be derived from the stored sections is derived here, then
// every record is decoded and every table entry is compared with what the decode
// finds.  Used after compression (self-check) and after deserialisation.
// --------------------------------------------------------------------------- //
int32_t finalize_and_validate(cl_layer *L)
{
    cl_layer_desc d = L->desc;
    if (int32_t rc = check_desc(d)) return rc;
    if (d.block_h != L->desc.block_h || d.block_w != L->desc.block_w || d.chunk_bits != L->desc.chunk_bits ||
        d.max_code_len != L->desc.max_code_len)
        return fail(CL_ECORRUPT, "descriptor is not in normal form");
    const Geometry g(d);
    const int nval = 1 << d.weight_bits, nidx = 1 << d.index_bits;
    L->n_blocks = g.n_blocks;
    L->n_panels = g.nbh;
    L->nbw = g.nbw;
    if ((int)L->codebook.size() != nval || (int)L->val_len.size() != nval || (int)L->idx_len.size() != nidx)
        return fail(CL_ECORRUPT, "codebook / code length tables have the wrong size");
    if (L->codebook[0] != 0.0f) return fail(CL_ECORRUPT, "codebook[0] must be 0");
    for (float c : L->codebook)
        if (!std::isfinite(c)) return fail(CL_ECORRUPT, "non-finite codebook entry");
    if (!canonical_codes(L->val_len, L->val_code, &L->val_lut_bits) ||
        !canonical_codes(L->idx_len, L->idx_code, &L->idx_lut_bits))
        return fail(CL_ECORRUPT, "code lengths are not a prefix code within the length limit");
    if (L->val_lut_bits > d.max_code_len || L->idx_lut_bits > d.max_code_len)
        return fail(CL_ECORRUPT, "code lengths exceed max_code_len");
    L->val_lut_bits = std::max(1, L->val_lut_bits);
    L->idx_lut_bits = std::max(1, L->idx_lut_bits);
    build_lut(L->val_len, L->val_code, L->val_lut_bits, L->val_lut);
    build_lut(L->idx_len, L->idx_code, L->idx_lut_bits, L->idx_lut);

    if ((int64_t)L->block_ptr.size() != g.n_blocks + 1) return fail(CL_ECORRUPT, "block_ptr has the wrong size");
    if ((int64_t)L->panel_chunk.size() != (int64_t)g.nbh + 1) return fail(CL_ECORRUPT, "panel table has the wrong size");
    if (L->meta.empty()) return fail(CL_ECORRUPT, "chunk table is empty");
    L->n_chunks = (int64_t)L->meta.size() - 1;
    L->n_records = (int64_t)L->records.size();
    L->entries = L->meta[L->n_chunks].sym_off;
    if (L->meta[L->n_chunks].rec_off != L->n_records) return fail(CL_ECORRUPT, "chunk table does not span the records");
    if (L->block_ptr[0] != 0 || L->block_ptr[g.n_blocks] != L->entries) return fail(CL_ECORRUPT, "block_ptr does not span the entries");
    for (int64_t b = 0; b < g.n_blocks; ++b)
        if (L->block_ptr[b] > L->block_ptr[b + 1]) return fail(CL_ECORRUPT, "block_ptr is not monotone");
    if (L->panel_chunk[0] != 0 || L->panel_chunk[g.nbh] != L->n_chunks) return fail(CL_ECORRUPT, "panel table does not span the chunks");
    L->max_panel_chunks = 0;
    for (int p = 0; p < g.nbh; ++p) {
        if (L->panel_chunk[p] > L->panel_chunk[p + 1]) return fail(CL_ECORRUPT, "panel table is not monotone");
        L->max_panel_chunks = std::max<int64_t>(L->max_panel_chunks, (int64_t)L->panel_chunk[p + 1] - L->panel_chunk[p]);
    }

    const uint32_t vmask = (1u << L->val_lut_bits) - 1u, imask = (1u << L->idx_lut_bits) - 1u;
    const uint32_t filler_z = (1u << d.index_bits) - 1u;
    int64_t nnz = 0, vbits = 0, ibits = 0;
    uint64_t next_entry = 0, next_rec = 0;
    int64_t cur_blk = -1;
    uint64_t possum = 0;
    int panel = 0;
    L->chunk_nz.assign((size_t)L->n_chunks + 1, 0u);
    for (int64_t c = 0; c < L->n_chunks; ++c) {
        const cl_chunk_meta &m = L->meta[c];
        L->chunk_nz[c] = (uint32_t)nnz;
        const uint64_t r0 = m.rec_off, r1 = L->meta[c + 1].rec_off;
        if (r0 != next_rec || r1 <= r0 || r1 - r0 > (uint64_t)kLanes || r1 > (uint64_t)L->n_records)
            return fail(CL_ECORRUPT, "chunk %lld: bad record range", (long long)c);
        if (m.sym_off != next_entry) return fail(CL_ECORRUPT, "chunk %lld: symbol offset is wrong", (long long)c);
        if (m.blk >= (uint64_t)g.n_blocks || (int64_t)m.blk < cur_blk) return fail(CL_ECORRUPT, "chunk %lld: bad block", (long long)c);
        if ((int64_t)m.blk != cur_blk) {
            if (m.sym_off != L->block_ptr[m.blk]) return fail(CL_ECORRUPT, "chunk %lld does not start its block", (long long)c);
            cur_blk = m.blk;
            possum = 0;
        }
        if (m.pos0 != possum) return fail(CL_ECORRUPT, "chunk %lld: position carry is wrong", (long long)c);
        while (panel < g.nbh && (int64_t)L->panel_chunk[panel + 1] <= c) ++panel;
        if ((int64_t)m.blk / g.nbw != panel) return fail(CL_ECORRUPT, "chunk %lld is not inside its block row", (long long)c);
        int row_id, col_id, bhp, bwp;
        g.block(m.blk, row_id, col_id, bhp, bwp);
        const uint64_t np = (uint64_t)bhp * bwp;
        for (uint64_t r = r0; r < r1; ++r) {
            const uint64_t w = L->records[r];
            const int n = (int)(w & 15u);
            if (n < 1) return fail(CL_ECORRUPT, "record %llu is empty", (unsigned long long)r);
            uint64_t vbuf = w >> kCountBits, ibuf = bit_reverse64(w);
            int vused = 0, iused = 0;
            for (int j = 0; j < n; ++j) {
                const lut_t ev = L->val_lut[(uint32_t)vbuf & vmask], ei = L->idx_lut[(uint32_t)ibuf & imask];
                const int v = lut_sym(ev), lv = lut_len(ev), z = lut_sym(ei), li = lut_len(ei);
                if (L->val_len[v] != lv || L->idx_len[z] != li) return fail(CL_ECORRUPT, "record %llu: bit pattern is not a codeword", (unsigned long long)r);
                vbuf >>= lv;
                ibuf >>= li;
                vused += lv;
                iused += li;
                if (kCountBits + vused + iused > CL_RECORD_BITS) return fail(CL_ECORRUPT, "record %llu overflows", (unsigned long long)r);
                possum += (uint64_t)z + 1;
                if (possum > np) return fail(CL_ECORRUPT, "record %llu: position leaves its block", (unsigned long long)r);
                if (v) ++nnz;
                else if ((uint32_t)z != filler_z) return fail(CL_ECORRUPT, "padding entry with a short gap");
            }
            // the bits between the two spans must be zero
            const int gap_bits = CL_RECORD_BITS - kCountBits - vused - iused;
            if (gap_bits > 0) {
                const uint64_t mid = (w >> (kCountBits + vused)) & ((gap_bits == 64 ? 0 : (1ull << gap_bits)) - 1ull);
                if (mid) return fail(CL_ECORRUPT, "record %llu: stray bits between its spans", (unsigned long long)r);
            }
            vbits += vused;
            ibits += iused;
            next_entry += (uint64_t)n;
        }
        if (next_entry > L->block_ptr[m.blk + 1]) return fail(CL_ECORRUPT, "chunk %lld runs past its block", (long long)c);
        next_rec = r1;
    }
    if (next_entry != (uint64_t)L->entries) return fail(CL_ECORRUPT, "records do not add up to the entry count");
    L->chunk_nz[L->n_chunks] = (uint32_t)nnz;
    // every non-empty block must have been covered in full
    for (int64_t c = 0; c < L->n_chunks; ++c) {
        const cl_chunk_meta &m = L->meta[c];
        const bool last_of_block = c + 1 == L->n_chunks || L->meta[c + 1].blk != m.blk;
        if (last_of_block && L->meta[c + 1].sym_off != L->block_ptr[m.blk + 1])
            return fail(CL_ECORRUPT, "block %u is not covered by its chunks", m.blk);
    }
    // first chunk of every block (blocks without entries get an empty range)
    L->block_chunk.assign((size_t)g.n_blocks + 1, (uint32_t)L->n_chunks);
    for (int64_t c = L->n_chunks - 1; c >= 0; --c) L->block_chunk[L->meta[c].blk] = (uint32_t)c;
    for (int64_t b = g.n_blocks - 1; b >= 0; --b)
        if (L->block_ptr[b] == L->block_ptr[b + 1]) L->block_chunk[b] = L->block_chunk[b + 1];
    L->max_block_nnz = 0;
    for (int64_t b = 0; b < g.n_blocks; ++b)
        L->max_block_nnz = std::max<int64_t>(L->max_block_nnz, (int64_t)L->chunk_nz[L->block_chunk[b + 1]] - L->chunk_nz[L->block_chunk[b]]);
    // the half-by-half order of the wide path (blocks of at most 128 x 128 only)
    L->chunk_half.clear();
    L->group_ptr.clear();
    if (d.block_h <= 128 && d.block_w <= 128) {
        constexpr int kGroups = 16, kPer = 2 * (kGroups + 1);
        L->chunk_half.assign((size_t)L->n_chunks * 2, 0u);
        L->group_ptr.assign((size_t)g.n_blocks * kPer, 0u);
        std::vector<uint32_t> cnt(2 * kGroups);
        for (int64_t b = 0; b < g.n_blocks; ++b) {
            const uint32_t c0 = L->block_chunk[b], c1 = L->block_chunk[b + 1];
            const uint32_t start = L->chunk_nz[c0];
            std::fill(cnt.begin(), cnt.end(), 0u);
            int row_id, col_id, bhp, bwp;
            g.block(b, row_id, col_id, bhp, bwp);
            uint32_t n[2] = {0, 0};
            for (uint32_t c = c0; c < c1; ++c) {
                L->chunk_half[2 * (size_t)c] = n[0];            // within the half for now
                L->chunk_half[2 * (size_t)c + 1] = n[1];
                uint64_t pos = L->meta[c].pos0;
                for (uint64_t r = L->meta[c].rec_off; r < L->meta[c + 1].rec_off; ++r) {
                    const uint64_t w = L->records[r];
                    uint64_t vbuf = w >> kCountBits, ibuf = bit_reverse64(w);
                    for (int j = 0, nj = (int)(w & 15u); j < nj; ++j) {
                        const lut_t ev = L->val_lut[(uint32_t)vbuf & vmask], ei = L->idx_lut[(uint32_t)ibuf & imask];
                        vbuf >>= lut_len(ev);
                        ibuf >>= lut_len(ei);
                        pos += (uint64_t)lut_sym(ei) + 1;
                        if (!lut_sym(ev)) continue;
                        const uint32_t at = (uint32_t)(pos - 1), row = at / (uint32_t)bwp, col = at % (uint32_t)bwp;
                        const int h = col >= 64 ? 1 : 0;
                        ++n[h];
                        ++cnt[(size_t)h * kGroups + (row >> 3)];
                    }
                }
            }
            for (uint32_t c = c0; c < c1; ++c) {
                L->chunk_half[2 * (size_t)c] += start;
                L->chunk_half[2 * (size_t)c + 1] += start + n[0];
            }
            uint32_t at = start;
            for (int h = 0; h < 2; ++h) {
                uint32_t *gp = &L->group_ptr[(size_t)b * kPer + (size_t)h * (kGroups + 1)];
                for (int q = 0; q < kGroups; ++q) {
                    gp[q] = at;
                    at += cnt[(size_t)h * kGroups + q];
                }
                gp[kGroups] = at;
            }
        }
    }
    L->max_group_blocks = 0;
    for (int p = 0; p < g.nbh; ++p)
        for (uint32_t c = L->panel_chunk[p]; c < L->panel_chunk[p + 1]; c += 8) {
            const uint32_t last = std::min<uint32_t>(c + 8, L->panel_chunk[p + 1]) - 1;
            L->max_group_blocks = std::max<int32_t>(L->max_group_blocks, (int32_t)(L->meta[last].blk - L->meta[c].blk) + 1);
        }
    L->nnz = nnz;
    L->padding = L->entries - nnz;
    L->val_bits = vbits;
    L->idx_bits = ibits;
    return CL_OK;
}

}  // namespace cl

using namespace cl;

extern "C" const char *cl_last_error(void) { return g_error.c_str(); }

extern "C" int32_t cl_compress_layer(const cl_layer_desc *desc, const float *W, const float *codebook_or_null,
                                     cl_layer **out)
{
    if (!desc || !W || !out) return fail(CL_EINVAL, "null argument");
    *out = nullptr;
    cl_layer_desc d = *desc;
    if (int32_t rc = check_desc(d)) return rc;
    const Geometry g(d);
    const int nval = 1 << d.weight_bits, nidx = 1 << d.index_bits, nc = nval - 1;
    const int64_t total = (int64_t)d.M * d.K;

    std::unique_ptr<cl_layer> L(new (std::nothrow) cl_layer);
    if (!L) return fail(CL_ENOMEM, "out of memory");
    try {
        L->desc = d;
        // ---- codebook (Sec. III-B: at most 2^r - 1 shared non-zero values plus 0) ----
        L->codebook.assign(nval, 0.0f);
        bool have = false;
        double lo = 0, hi = 0;
        for (int64_t i = 0; i < total; ++i) {
            const float w = W[i];
            if (!std::isfinite(w)) return fail(CL_EINVAL, "non-finite weight at element %lld", (long long)i);
            if (w == 0.0f) continue;
            if (!have) { lo = hi = w; have = true; }
            else { lo = std::min(lo, (double)w); hi = std::max(hi, (double)w); }
        }
        if (codebook_or_null) {
            if (codebook_or_null[0] != 0.0f) return fail(CL_EINVAL, "codebook[0] must be 0");
            for (int t = 0; t < nval; ++t) {
                if (!std::isfinite(codebook_or_null[t])) return fail(CL_EINVAL, "non-finite codebook entry");
                L->codebook[t] = codebook_or_null[t];
            }
        } else if (have) {
            for (int t = 1; t <= nc; ++t)
                L->codebook[t] = (float)(nc == 1 ? 0.5 * (lo + hi) : lo + (double)(t - 1) * (hi - lo) / (double)(nc - 1));
        }
        // ---- value index of every surviving weight: nearest centre, ties to the lower index ----
        std::vector<uint8_t> q((size_t)total, 0);
        std::vector<double> centre(nval);
        for (int t = 0; t < nval; ++t) centre[t] = (double)L->codebook[t];
        for (int64_t i = 0; i < total; ++i) {
            if (W[i] == 0.0f) continue;
            const double w = (double)W[i];
            int best = 1;
            double bd = std::fabs(w - centre[1]);
            for (int t = 2; t <= nc; ++t) {
                const double dd = std::fabs(w - centre[t]);
                if (dd < bd) { bd = dd; best = t; }
            }
            q[(size_t)i] = (uint8_t)best;
        }
        // ---- relative-indexed entries, block after block, row by row inside a block ----
        const int R = 1 << d.index_bits;
        std::vector<uint8_t> val, idx;
        val.reserve((size_t)(total / 8 + 16));
        idx.reserve((size_t)(total / 8 + 16));
        L->block_ptr.assign((size_t)g.n_blocks + 1, 0);
        for (int64_t b = 0; b < g.n_blocks; ++b) {
            int row_id, col_id, bhp, bwp;
            g.block(b, row_id, col_id, bhp, bwp);
            L->block_ptr[(size_t)b] = (uint32_t)val.size();
            int64_t run = 0;   // zeros seen since the last stored element
            for (int r = 0; r < bhp; ++r) {
                const uint8_t *row = q.data() + (size_t)(row_id + r) * d.K + col_id;
                for (int c = 0; c < bwp; ++c) {
                    const uint8_t s = row[c];
                    if (!s) { ++run; continue; }
                    while (run >= R) { val.push_back(0); idx.push_back((uint8_t)(R - 1)); run -= R; }
                    val.push_back(s);
                    idx.push_back((uint8_t)run);
                    run = 0;
                }
            }
            if (val.size() > (size_t)std::numeric_limits<int32_t>::max()) return fail(CL_EINVAL, "more than 2^31-1 entries");
        }
        L->block_ptr[(size_t)g.n_blocks] = (uint32_t)val.size();
        const int64_t n_entries = (int64_t)val.size();
        q.clear();
        q.shrink_to_fit();
        // ---- Huffman codes of the two arrays ----
        std::vector<int64_t> vcount(nval, 0), icount(nidx, 0);
        for (int64_t e = 0; e < n_entries; ++e) { ++vcount[val[(size_t)e]]; ++icount[idx[(size_t)e]]; }
        if (!limited_code_lengths(vcount, d.max_code_len, L->val_len) || !limited_code_lengths(icount, d.max_code_len, L->idx_len))
            return fail(CL_EINVAL, "alphabet does not fit max_code_len");
        L->val_bits_unlimited = unlimited_code_bits(vcount);
        L->idx_bits_unlimited = unlimited_code_bits(icount);
        int dummy;
        if (!canonical_codes(L->val_len, L->val_code, &dummy) || !canonical_codes(L->idx_len, L->idx_code, &dummy))
            return fail(CL_EINVAL, "internal: code construction failed");
        // ---- lane records and chunks: a record takes as many whole entries as fit its 64 bits,
        // a chunk takes up to 64 records; neither crosses a block ----
        L->panel_chunk.assign((size_t)g.nbh + 1, 0);
        for (int64_t b = 0; b < g.n_blocks; ++b) {
            if (b % g.nbw == 0) L->panel_chunk[(size_t)(b / g.nbw)] = (uint32_t)L->meta.size();
            const int64_t be0 = L->block_ptr[(size_t)b], be1 = L->block_ptr[(size_t)b + 1];
            uint64_t possum = 0;
            int in_chunk = kLanes;
            for (int64_t e = be0; e < be1;) {
                if (in_chunk == kLanes) {
                    cl_chunk_meta m;
                    m.sym_off = (uint32_t)e;
                    m.rec_off = (uint32_t)L->records.size();
                    m.blk = (uint32_t)b;
                    m.pos0 = (uint32_t)possum;
                    L->meta.push_back(m);
                    in_chunk = 0;
                }
                uint64_t rec = 0;
                int vpos = kCountBits, itop = CL_RECORD_BITS, n = 0;     // value bits go up from vpos, index bits down from itop
                while (e + n < be1 && n < CL_MAX_RECORD_ENTRIES) {
                    const uint8_t v = val[(size_t)(e + n)], z = idx[(size_t)(e + n)];
                    const int lv = L->val_len[v], li = L->idx_len[z];
                    if (vpos + lv + li > itop) break;
                    rec |= (uint64_t)L->val_code[v] << vpos;
                    vpos += lv;
                    for (int j = 0; j < li; ++j)
                        rec |= (uint64_t)((L->idx_code[z] >> j) & 1u) << (itop - 1 - j);
                    itop -= li;
                    possum += (uint64_t)z + 1;
                    ++n;
                }
                rec |= (uint64_t)n;
                L->records.push_back(rec);
                e += n;
                ++in_chunk;
            }
        }
        L->panel_chunk[(size_t)g.nbh] = (uint32_t)L->meta.size();
        cl_chunk_meta sentinel{};
        sentinel.sym_off = (uint32_t)n_entries;
        sentinel.rec_off = (uint32_t)L->records.size();
        L->meta.push_back(sentinel);
    } catch (const std::bad_alloc &) {
        return fail(CL_ENOMEM, "out of memory");
    }
    const int64_t vu = L->val_bits_unlimited, iu = L->idx_bits_unlimited;
    if (int32_t rc = finalize_and_validate(L.get())) return fail(rc == CL_ECORRUPT ? CL_EINVAL : rc, "internal: self-check failed: %s", cl_last_error());
    L->val_bits_unlimited = vu;
    L->idx_bits_unlimited = iu;
    *out = L.release();
    clear_error();
    return CL_OK;
}

extern "C" int32_t cl_layer_free(cl_layer *layer)
{
    if (!layer) return CL_OK;
    release_device(layer);
    delete layer;
    return CL_OK;
}

extern "C" int32_t cl_layer_stats(const cl_layer *L, cl_stats *s)
{
    if (!L || !s) return fail(CL_EINVAL, "null argument");
    std::memset(s, 0, sizeof *s);
    s->nnz = L->nnz;
    s->padding = L->padding;
    s->entries = L->entries;
    s->n_blocks = L->n_blocks;
    s->n_chunks = L->n_chunks;
    s->val_bits = L->val_bits;
    s->idx_bits = L->idx_bits;
    s->val_bits_unlimited = L->val_bits_unlimited;
    s->idx_bits_unlimited = L->idx_bits_unlimited;
    s->n_records = L->n_records;
    s->payload_bytes = L->n_records * 8;
    s->table_bytes = (int64_t)(L->meta.size() * sizeof(cl_chunk_meta) + L->block_ptr.size() * 4 + L->panel_chunk.size() * 4);
    s->model_bytes = s->payload_bytes + s->table_bytes + (int64_t)(L->codebook.size() * 4 + L->val_len.size() + L->idx_len.size());
    s->lut_bytes = (int64_t)((L->val_lut.size() + L->idx_lut.size()) * sizeof(lut_t));
    s->val_max_len = L->val_lut_bits;
    s->idx_max_len = L->idx_lut_bits;
    return CL_OK;
}

extern "C" int32_t cl_layer_host_view(const cl_layer *L, cl_host_view *v)
{
    if (!L || !v) return fail(CL_EINVAL, "null argument");
    v->desc = L->desc;
    v->codebook = L->codebook.data();
    v->val_len = L->val_len.data();
    v->val_code = L->val_code.data();
    v->idx_len = L->idx_len.data();
    v->idx_code = L->idx_code.data();
    v->block_ptr = L->block_ptr.data();
    v->panel_chunk = L->panel_chunk.data();
    v->chunk_meta = L->meta.data();
    v->chunk_nz = L->chunk_nz.data();
    v->max_block_nnz = L->max_block_nnz;
    v->max_group_blocks = L->max_group_blocks;
    v->chunk_half = L->chunk_half.empty() ? nullptr : L->chunk_half.data();
    v->group_ptr = L->group_ptr.empty() ? nullptr : L->group_ptr.data();
    v->records = L->records.data();
    v->n_blocks = L->n_blocks;
    v->n_chunks = L->n_chunks;
    v->n_records = L->n_records;
    v->n_entries = L->entries;
    v->n_panels = L->n_panels;
    return CL_OK;
}

// --------------------------------------------------------------------------- //
// Byte image: header, then the stored sections back to back (little endian).
// --------------------------------------------------------------------------- //
namespace {
struct ImageHeader {
    char magic[8];          // "CLZLAYER"
    uint32_t version;
    uint32_t header_bytes;
    cl_layer_desc desc;
    int64_t n_blocks, n_chunks, n_records, n_entries;
    int64_t val_bits_unlimited, idx_bits_unlimited;
    uint64_t checksum;      // FNV-1a over every byte after the header
};
uint64_t fnv1a(const void *data, size_t n)
{
    const uint8_t *p = (const uint8_t *)data;
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < n; ++i) { h ^= p[i]; h *= 1099511628211ull; }
    return h;
}
const char kMagic[8] = {'C', 'L', 'Z', 'L', 'A', 'Y', 'E', 'R'};

template <class T>
size_t section_bytes(const std::vector<T> &v) { return v.size() * sizeof(T); }
}  // namespace

extern "C" int32_t cl_layer_serialize(const cl_layer *L, void *buf, size_t *bytes)
{
    if (!L || !bytes) return fail(CL_EINVAL, "null argument");
    const size_t need = sizeof(ImageHeader) + section_bytes(L->codebook) + section_bytes(L->val_len) +
                        section_bytes(L->idx_len) + section_bytes(L->block_ptr) + section_bytes(L->panel_chunk) +
                        section_bytes(L->meta) + section_bytes(L->records);
    if (!buf) { *bytes = need; return CL_OK; }
    if (*bytes < need) { *bytes = need; return fail(CL_EINVAL, "buffer too small: need %zu bytes", need); }
    ImageHeader h{};
    std::memcpy(h.magic, kMagic, 8);
    h.version = 2;
    h.header_bytes = sizeof(ImageHeader);
    h.desc = L->desc;
    h.n_blocks = L->n_blocks;
    h.n_chunks = L->n_chunks;
    h.n_records = L->n_records;
    h.n_entries = L->entries;
    h.val_bits_unlimited = L->val_bits_unlimited;
    h.idx_bits_unlimited = L->idx_bits_unlimited;
    char *p = (char *)buf + sizeof h;
    auto put = [&](const void *src, size_t n) { if (n) std::memcpy(p, src, n); p += n; };
    put(L->codebook.data(), section_bytes(L->codebook));
    put(L->val_len.data(), section_bytes(L->val_len));
    put(L->idx_len.data(), section_bytes(L->idx_len));
    put(L->block_ptr.data(), section_bytes(L->block_ptr));
    put(L->panel_chunk.data(), section_bytes(L->panel_chunk));
    put(L->meta.data(), section_bytes(L->meta));
    put(L->records.data(), section_bytes(L->records));
    h.checksum = fnv1a((const char *)buf + sizeof h, need - sizeof h);
    std::memcpy(buf, &h, sizeof h);
    *bytes = need;
    return CL_OK;
}

extern "C" int32_t cl_layer_deserialize(const void *buf, size_t bytes, cl_layer **out)
{
    if (!buf || !out) return fail(CL_EINVAL, "null argument");
    *out = nullptr;
    if (bytes < sizeof(ImageHeader)) return fail(CL_ECORRUPT, "image shorter than its header");
    ImageHeader h;
    std::memcpy(&h, buf, sizeof h);
    if (std::memcmp(h.magic, kMagic, 8) || h.version != 2 || h.header_bytes != sizeof(ImageHeader))
        return fail(CL_ECORRUPT, "not a compressed-layer image");
    cl_layer_desc d = h.desc;
    if (check_desc(d) != CL_OK) return fail(CL_ECORRUPT, "bad descriptor: %s", cl_last_error());
    const Geometry g(d);
    if (h.n_blocks != g.n_blocks || h.n_chunks < 0 || h.n_entries < 0 || h.n_chunks > h.n_records || h.n_records > h.n_entries ||
        h.n_entries > std::numeric_limits<int32_t>::max())
        return fail(CL_ECORRUPT, "inconsistent counts");
    const size_t nval = (size_t)1 << d.weight_bits, nidx = (size_t)1 << d.index_bits;
    const size_t need = sizeof(ImageHeader) + nval * 4 + nval + nidx + ((size_t)g.n_blocks + 1) * 4 + ((size_t)g.nbh + 1) * 4 +
                        ((size_t)h.n_chunks + 1) * sizeof(cl_chunk_meta) + (size_t)h.n_records * 8;
    if (bytes != need) return fail(CL_ECORRUPT, "image size %zu does not match its header (%zu)", bytes, need);
    if (fnv1a((const char *)buf + sizeof h, need - sizeof h) != h.checksum) return fail(CL_ECORRUPT, "checksum mismatch");
    std::unique_ptr<cl_layer> L(new (std::nothrow) cl_layer);
    if (!L) return fail(CL_ENOMEM, "out of memory");
    try {
        L->desc = h.desc;
        const char *p = (const char *)buf + sizeof(ImageHeader);
        auto get = [&](auto &vec, size_t n) {
            vec.resize(n);
            if (n) std::memcpy(vec.data(), p, n * sizeof(vec[0]));
            p += n * sizeof(vec[0]);
        };
        get(L->codebook, nval);
        get(L->val_len, nval);
        get(L->idx_len, nidx);
        get(L->block_ptr, (size_t)g.n_blocks + 1);
        get(L->panel_chunk, (size_t)g.nbh + 1);
        get(L->meta, (size_t)h.n_chunks + 1);
        get(L->records, (size_t)h.n_records);
    } catch (const std::bad_alloc &) {
        return fail(CL_ENOMEM, "out of memory");
    }
    if (L->meta[(size_t)h.n_chunks].sym_off != (uint64_t)h.n_entries) return fail(CL_ECORRUPT, "entry count mismatch");
    if (int32_t rc = finalize_and_validate(L.get())) return rc;
    L->val_bits_unlimited = h.val_bits_unlimited;
    L->idx_bits_unlimited = h.idx_bits_unlimited;
    *out = L.release();
    clear_error();
    return CL_OK;
}
