// Internal representation of a compressed layer (host copy + device image).
#pragma once
#include <cstdarg>
#include <cstdint>
#include <string>
#include <vector>

#include "compressed_layer.h"

namespace cl {

constexpr int kLanes = CL_RECORDS_PER_CHUNK;        // one 64-bit record per lane of a wavefront
constexpr int kCountBits = 4;                       // width of a record's entry-count field

int32_t fail(int32_t code, const char *fmt, ...);
void clear_error();

// Entry of a decode table: low byte = codeword length (>= 1, <= CL_MAX_CODE_LEN, so
// the entry can feed a 64-bit shift, which looks at the low six bits only), next byte
// = symbol.
constexpr int lut_len(uint16_t e) { return e & 0xff; }
constexpr int lut_sym(uint16_t e) { return e >> 8; }
using lut_t = uint16_t;

struct DeviceImage {
    int device = -1;
    char *blob = nullptr;          // one allocation; the pointers below point into it
    size_t blob_bytes = 0;
    const uint64_t *records = nullptr;
    const cl_chunk_meta *meta = nullptr;
    const uint32_t *block_ptr = nullptr;
    const uint32_t *panel_chunk = nullptr;
    const uint32_t *block_chunk = nullptr;
    const uint32_t *chunk_nz = nullptr;
    const uint32_t *chunk_half = nullptr;
    const uint32_t *group_ptr = nullptr;
    const float *codebook = nullptr;
    const lut_t *val_lut = nullptr;
    const lut_t *idx_lut = nullptr;
};

}  // namespace cl

struct cl_layer {
    cl_layer_desc desc{};
    int64_t nnz = 0, padding = 0, entries = 0, n_blocks = 0, n_chunks = 0, n_records = 0;
    int32_t n_panels = 0;          // block rows
    int32_t nbw = 0;               // blocks across
    int64_t max_panel_chunks = 0;  // most chunks in any block row
    int64_t val_bits = 0, idx_bits = 0, val_bits_unlimited = 0, idx_bits_unlimited = 0;
    std::vector<float> codebook;
    std::vector<uint8_t> val_len, idx_len;
    std::vector<uint32_t> val_code, idx_code;       // codewords, bit j = j-th bit in tree-walk order
    std::vector<uint32_t> block_ptr, panel_chunk;
    std::vector<uint32_t> block_chunk;              // n_blocks + 1: first chunk of each block (derived)
    std::vector<uint32_t> chunk_nz;                 // n_chunks + 1: surviving weights (entries that are not padding) in all
                                                    //   chunks before this one (derived)
    int64_t max_block_nnz = 0;                      // most surviving weights in one block
    int32_t max_group_blocks = 0;                   // most blocks touched by eight consecutive chunks of a block row that start
                                                    //   at a multiple of eight from the block row's first (the share of one
                                                    //   workgroup of the small-batch kernel)
    // For layers whose blocks are at most 128 x 128 (else empty), the order in which the wide
    // path lists a block's surviving weights: first those in the block's columns 0-63, then
    // those in columns 64-127, each half row by row (derived).
    std::vector<uint32_t> chunk_half;               // 2 n_chunks: where in that list the chunk's first surviving weight of
                                                    //   each half goes
    std::vector<uint32_t> group_ptr;                // n_blocks x 2 x 17: where each group of eight rows starts in each
                                                    //   half of the block's part of the list, and where the half ends
    std::vector<cl_chunk_meta> meta;                // n_chunks + 1
    std::vector<uint64_t> records;
    std::vector<cl::lut_t> val_lut, idx_lut;        // indexed by the next val_lut_bits / idx_lut_bits stream bits
    int val_lut_bits = 1, idx_lut_bits = 1;         // longest codeword of each code
    cl::DeviceImage dev;
};

namespace cl {

// huffman.cpp
// Optimal prefix-code lengths under a length limit (package-merge).  counts[s] == 0
// gives len[s] == 0.  Returns false when 2^limit < number of used symbols.
bool limited_code_lengths(const std::vector<int64_t> &counts, int limit, std::vector<uint8_t> &len);
// Coded size under an unrestricted Huffman code (sum of merged weights).
int64_t unlimited_code_bits(const std::vector<int64_t> &counts);
// Canonical codewords from lengths (bit j = j-th bit written).  Returns false when
// the lengths violate Kraft's inequality or exceed CL_MAX_CODE_LEN.
bool canonical_codes(const std::vector<uint8_t> &len, std::vector<uint32_t> &code, int *max_len);
// Flat decode table indexed by the next max_len stream bits.
void build_lut(const std::vector<uint8_t> &len, const std::vector<uint32_t> &code, int max_len,
               std::vector<lut_t> &lut);

// compress.cpp
// Derive codes and decode tables from the stored lengths, then decode every record
// on the host and check every table against what the decode finds.
int32_t finalize_and_validate(cl_layer *L);

// device.hip
void release_device(cl_layer *L);

}  // namespace cl
