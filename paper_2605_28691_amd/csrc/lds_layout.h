// LDS layouts of a staged tile of 64 rows of head_dim bf16 (or 8-bit) values, shared by the attention kernels.
//
// Tiles arrive through global_load_lds_dwordx4, which writes the 64 lanes' 16-byte chunks to 64 consecutive chunk positions, so
// rows are packed (row r starts at r * 2*D bytes) and there is no room for padding.  Bank conflicts are avoided by storing chunk
// c of row r at chunk position c ^ lds_swizzle<D>(r).  The function only looks at the low four bits of r, and is chosen so that
//   * the 16-byte fragment reads of 16 consecutive rows (one MFMA A-operand read per 16 lanes), and
//   * the transposing reads (ds_read_b64_tr_b16) of 4 consecutive rows x 64 bytes (32 lanes)
// each touch every one of the 64 banks exactly once.
#pragma once
#include <stdint.h>

namespace skiparse {

template <int D>
__host__ __device__ constexpr uint32_t lds_swizzle(uint32_t r) {
    static_assert(D == 64 || D == 128, "head_dim");
    // D = 128: 16 chunks per 256-byte row (one row spans all banks): rows r..r+3 get different 64-byte groups (bits 2-3), rows
    //          that differ in bits 2-3 get different chunks inside the group.
    // D = 64:  8 chunks per 128-byte row, two rows per pass over the banks: the pair index r>>1 is spread over the 8 positions.
    return D == 128 ? (((r & 3u) << 2) | ((r >> 2) & 3u)) : ((((r >> 1) & 1u) << 2) | ((r >> 2) & 3u));
}

// The same for a tile of 64 rows of head_dim 8-bit values (the fp8 kernel): chunk c of row r sits at chunk position
// c ^ lds_swizzle8<D>(r).  head_dim 128: 8 chunks per row, two rows per pass over the banks; head_dim 64: 4 chunks per row, four rows
// per pass.  Conflict-free for the 16-byte fragment reads of 16 consecutive rows and for the transposing byte reads
// (ds_read_b64_tr_b8: 8 consecutive rows x 32 bytes per 32 lanes).
template <int D>
__host__ __device__ constexpr uint32_t lds_swizzle8(uint32_t r) {
    static_assert(D == 64 || D == 128, "head_dim");
    return D == 128 ? ((((r >> 1) & 3u) << 1) | ((r >> 3) & 1u)) : ((((r >> 2) & 1u) << 1) | ((r >> 3) & 1u));
}

}  // namespace skiparse
