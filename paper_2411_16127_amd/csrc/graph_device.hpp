// Device helpers and counter slots shared by the two graph-metadata builders (graph.hip: any graph, many
// launches; graph_local.hip: small graphs and batches of small graphs, one to three launches).
#pragma once
#include "common.hpp"

namespace dfgnn {

// words of the device counter block inside the metadata buffer (read back by the host in one copy)
enum { CNT_ROW_CHUNKS = 1, CNT_COL_CHUNKS = 3, CNT_NEAR = 4, CNT_ERROR = 8, CNT_BATCH = 9, CNT_BATCH_MAX = 10,
       CNT_BATCH_PAIRS = 12, CNT_N_TILES = 14, CNT_SEG_FLAGS = 15, CNT_ROW_BUCKETS = 16, CNT_COL_BUCKETS = 56, CNT_TOTAL = 96 };
// bits of counter CNT_ERROR (malformed CSR)
enum { CSR_FIRST_NOT_ZERO = 1, CSR_LAST_NOT_E = 2, CSR_DECREASES = 4, CSR_PTR_RANGE = 8, CSR_INDEX_RANGE = 16 };
// bits of counter CNT_BATCH
enum { BATCH_BAD_PTR = 1, BATCH_CROSS_EDGE = 2, BATCH_TOO_LARGE = 4, BATCH_DUPLICATE = 8 };

constexpr int kLocalityWindow = 4096;  // |row - source| below which an edge counts as local in the numbering

// sort key of a row (or column) of `deg` entries: 0 for super rows, else 33 - bit_length(deg), so that
// long rows sort before short ones
__device__ inline uint32_t degree_key(int deg, int T) { return deg >= T ? 0u : (uint32_t)(33 - (32 - __clz(deg))); }

// lanes of the wave whose (valid) digit equals this lane's digit; BITS = width of a digit
template <int BITS = 8> __device__ inline unsigned long long match_digit(unsigned d, bool valid) {
    unsigned long long mask = __ballot(valid);
#pragma unroll
    for (int b = 0; b < BITS; ++b) {
        const bool bit = (d >> b) & 1u;
        const unsigned long long bal = __ballot(valid && bit);
        mask &= bit ? bal : ~bal;
    }
    return mask;
}

}  // namespace dfgnn
