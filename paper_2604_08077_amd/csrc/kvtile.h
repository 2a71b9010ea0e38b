// Packed KV layout shared by kv_pack_kernel (writer) and the attention kernels (readers).
//
// Per KV head, per cube, per 64-key tile the workspace holds
//     K tile : 64 rows (keys, rank order) x D bf16
//     V^T tile: D rows x 64 keys bf16 (transposed: the P.V MFMA operand is 16 contiguous bytes)
// each tile contiguous (64*D*2 bytes).  Inside a tile the 16-byte chunks of a row are XOR-swizzled so that
// a linear copy of the tile into LDS can be read by the MFMA operand loads without bank conflicts:
// the 16 lanes that read the same logical chunk of 16 different rows land on 16 different 16-byte slots of a
// 256-byte LDS line.  Cubes are padded to a whole number of tiles with zero keys / zero values.
#pragma once
#include "geom.h"

namespace adaspark {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // a 16-byte chunk in registers

// Byte offset, inside a K tile, of 16-byte chunk `chunk` (8 head-dim elements) of key row `row`.
template <int D>
__host__ __device__ inline int k_tile_off(int row, int chunk)
{
    if (D == 128) {  // 256-byte rows, 16 chunks
        return row * 256 + ((chunk ^ ((((row >> 3) & 3) << 2) | (row & 3))) << 4);
    } else {  // 128-byte rows: two rows share a 256-byte line of 16 slots
        const int slot = ((row & 1) << 3) | chunk;
        const int x = (((row >> 3) & 3) << 1) | ((row >> 1) & 1);
        return (row >> 1) * 256 + ((slot ^ x) << 4);
    }
}

// Byte offset, inside a V^T tile, of 16-byte chunk `chunk` (8 keys) of head-dim row `d` (rows are 128 bytes).
__host__ __device__ inline int vt_tile_off(int d, int chunk)
{
    const int slot = ((d & 1) << 3) | chunk;
    return (d >> 1) * 256 + ((slot ^ ((d >> 1) & 7)) << 4);
}

// Inverse maps: physical 16-byte slot x of a tile (x = byte offset / 16) -> logical (row, chunk).
template <int D>
__host__ __device__ inline void k_tile_coords(int x, int &row, int &chunk)
{
    if (D == 128) {
        row = x >> 4;
        chunk = (x & 15) ^ ((((row >> 3) & 3) << 2) | (row & 3));
    } else {
        const int line = x >> 4;
        // the XOR value depends only on bits of the row above bit 0, i.e. on the line
        const int slot = (x & 15) ^ ((((line >> 2) & 3) << 1) | (line & 1));
        row = (line << 1) | (slot >> 3);
        chunk = slot & 7;
    }
}
__host__ __device__ inline void vt_tile_coords(int x, int &d, int &chunk)
{
    const int line = x >> 4;
    const int slot = (x & 15) ^ (line & 7);
    d = (line << 1) | (slot >> 3);
    chunk = slot & 7;
}

template <int D>
__host__ __device__ inline size_t kv_tile_bytes() { return (size_t)KEY_TILE * D * 2; }

}  // namespace adaspark
