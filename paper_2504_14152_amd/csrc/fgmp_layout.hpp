// Packed storage of an FGMP tensor (rows x K, 16-element blocks along K).
//
// The paper fixes the content of a block -- 16 E2M1 nibbles plus one E4M3
// scale, or 16 E4M3 bytes and no scale, plus one metadata bit (Sec. 4,
// Sec. 5.1, Sec. 5.4.1) -- but not how the unstructured mix is laid out in
// memory.  This layout is made for coalesced 64-lane access on gfx950:
//
//   tile      8 rows x 128 K-elements = 64 blocks, one block per lane of a
//             wavefront: slot j = (row j/8, K-block j%8) of the tile.
//             Tiles are ordered row-tile major: t = rt * n_kt + kt.
//   plane L   8 bytes per slot (512 B per tile): the 16 E2M1 nibbles of an
//             FP4 block (element 2i in the low nibble of byte i), or the
//             first 8 E4M3 bytes of an FP8 block.
//   plane S   1 byte per slot (64 B per tile): the E4M3 block scale of an FP4
//             block; for an FP8 block, which has no scale, the index of its
//             entry among the tile's entries in plane H -- the number of FP8
//             slots before it in the tile (readers may take it from the mask).
//   plane M   one 64-bit word per tile: bit j set = slot j is FP8.
//   plane T   one uint32 per tile: index (in 8-byte entries) of the tile's
//             first entry in plane H.
//   plane H   8 bytes per FP8 block: its last 8 E4M3 bytes.  "strided"
//             tensors (activations, written in one pass) reserve room for 64
//             entries per tile; where a tile's entries start is the writer's
//             choice (T[t] = 64 t, or the tiles one wave visits appended one
//             after the other) and readers only go by T[t].  "compact" tensors
//             (weights, packed offline) store the entries back to back in tile
//             order -- T[t + 1] = T[t] + number of FP8 slots of tile t -- so
//             the tensor occupies 9 B per FP4 block and 16 B per FP8 block
//             plus tables.
//   Slots outside the tensor (row >= rows or K-block >= K/16) hold FP4 zeros.
//
// A 256-byte header precedes the planes; every plane starts 256-byte aligned.
#pragma once
#include <stdint.h>

namespace fgmp {

constexpr int kBlock = 16;        // elements per block (Sec. 4)
constexpr int kTileRows = 8;
constexpr int kTileBlocks = 8;    // K-blocks per tile row
constexpr int kTileK = kTileBlocks * kBlock;  // 128
constexpr int kTileSlots = kTileRows * kTileBlocks;  // 64
constexpr uint32_t kMagic = 0x504D4746u;  // "FGMP"
constexpr uint32_t kVersion = 1;
constexpr int64_t kHeaderBytes = 256;

struct PackedHeader {
    uint32_t magic, version;
    int64_t rows, K;
    float tensor_scale;
    uint32_t compact;
    uint64_t off_L, off_S, off_M, off_T, off_H;
    uint64_t h_entries;   // entries of plane H in use (compact) or reserved (strided)
    uint64_t bytes_used;  // header + planes up to the last byte a reader may touch
};
static_assert(sizeof(PackedHeader) <= kHeaderBytes, "header too large");

struct PackedLayout {
    int64_t rows, K;
    int64_t nb;            // K / 16
    int64_t n_rt, n_kt, n_tiles;
    uint64_t off_L, off_S, off_M, off_T, off_H, total_bytes;
};

__host__ __device__ inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

__host__ __device__ inline PackedLayout make_layout(int64_t rows, int64_t K)
{
    PackedLayout l;
    l.rows = rows;
    l.K = K;
    l.nb = K / kBlock;
    l.n_rt = (rows + kTileRows - 1) / kTileRows;
    l.n_kt = (l.nb + kTileBlocks - 1) / kTileBlocks;
    l.n_tiles = l.n_rt * l.n_kt;
    uint64_t nt = (uint64_t)l.n_tiles;
    l.off_L = kHeaderBytes;
    l.off_S = align_up(l.off_L + nt * kTileSlots * 8, 256);
    l.off_M = align_up(l.off_S + nt * kTileSlots, 256);
    l.off_T = align_up(l.off_M + nt * 8, 256);
    l.off_H = align_up(l.off_T + nt * 4, 256);
    l.total_bytes = align_up(l.off_H + nt * kTileSlots * 8, 256);
    return l;
}

// Device-side view of a packed tensor's planes.
struct PackedView {
    uint2 *L;        // [n_tiles][64]
    uint8_t *S;      // [n_tiles][64]
    uint64_t *M;     // [n_tiles]
    uint32_t *T;     // [n_tiles]
    uint2 *H;        // entries
    PackedHeader *hdr;
};

inline PackedView make_view(void *base, const PackedLayout &l)
{
    char *p = static_cast<char *>(base);
    PackedView v;
    v.hdr = reinterpret_cast<PackedHeader *>(p);
    v.L = reinterpret_cast<uint2 *>(p + l.off_L);
    v.S = reinterpret_cast<uint8_t *>(p + l.off_S);
    v.M = reinterpret_cast<uint64_t *>(p + l.off_M);
    v.T = reinterpret_cast<uint32_t *>(p + l.off_T);
    v.H = reinterpret_cast<uint2 *>(p + l.off_H);
    return v;
}

}  // namespace fgmp
