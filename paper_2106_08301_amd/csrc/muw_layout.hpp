// muw_layout.hpp -- private device layout of an encoded layer and the per-lane decode of it.
//
// Geometry (chosen for 64-wide wavefronts and the 16x16x32 bf16 MFMA):
//   strip  = 16 consecutive output rows n
//   panel  = one strip x 64 consecutive k             (two 16x16x32 MFMA B-operands)
//   tile   = one strip x 256 consecutive k = up to 4 panels; the unit that owns payload streams
// Inside a panel, lane l = (r = l % 16, g = l / 16) owns row r and the 16 weights k = 16 g .. 16 g + 15
// of the panel, i.e. S = 16 / B whole blocks ("sub-steps" j = 0 .. S-1, block column S*g + j of the
// panel).  MFMA h (h = 0, 1) of the panel takes the lane's weights 8 h .. 8 h + 7, so the matching
// activation operand of lane (m, g) is X[m][64 p + 16 g + 8 h .. + 7]: one 16-byte load.
//
// A tile's byte stream (16-byte aligned, padded to 16 bytes):
//   masks   per panel: U[0..S-1] then D[0..S-1], 64-bit each; bit l of U[j] / D[j] says that lane l's
//           block j is UNIFIED / DENSE.  Neither bit: PRUNED (or outside the matrix).  2 bits per block.
//           The mask area always spans 4 panels (a ragged last tile has zero masks for the panels it
//           lacks), so payload offsets do not depend on the tile's position.
//   mags    one stored magnitude per UNIFIED block, in (panel, sub-step, lane) order
//   signs   B bits per UNIFIED block, same order, bit-packed; inside a block the bits are permuted
//           (sign_pos) so that the bf16 decode is one shift and one bit-select per output dword
//           (B = 16 with bf16 storage: mags and signs are interleaved instead, one 32-bit record per
//           UNIFIED block, bytes {magnitude low, sign field low, magnitude high, sign field high}: a
//           block costs a single 4-byte read and the record itself is the sign word of the decode --
//           bits 15 - d and 31 - d hold the signs of elements 2 d and 2 d + 1, see pack_record16)
//   dense   the B values of each DENSE block, same order, starting at the next multiple of 16 bytes
//   Masks first and dense last: every offset inside a tile, and the tile's size, follow from the
//   popcounts of its masks alone (the streaming kernel never needs the directory to decode).
// Because payload order is (panel, sub-step, lane), the payload index of a lane's block is the
// running count of earlier blocks plus the popcount of the mask below the lane (v_mbcnt): PRUNED
// blocks cost 2 mask bits and nothing else (Sec. 3.1: storage of pruned blocks is skipped).
//
// Blob = [64-byte header][directory: (NT + 1) x {u32 offset/16, u16 nU, u16 nD}][tile streams],
// tiles ordered strip-major so that one strip's K range is contiguous in memory.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace muw {

constexpr int kStripRows = 16;
constexpr int kPanelK = 64;
constexpr int kTilePanels = 4;
constexpr int kTileK = kPanelK * kTilePanels;
constexpr uint32_t kMagic = 0x3157554du;  // "MUW1"
constexpr size_t kHeaderBytes = 64;

struct DirEntry {
    uint32_t off16;  // tile stream offset from the start of the stream area, in 16-byte units
    uint16_t nU;     // UNIFIED blocks in the tile
    uint16_t nD;     // DENSE blocks in the tile
};

struct Layout {
    int64_t N, K;
    int32_t B, vb;       // block length, value bytes (2 = bf16, 4 = fp32)
    int32_t S;           // sub-steps per panel = 16 / B
    int64_t KB;          // blocks per row
    int64_t NS, KP, KT;  // strips, panels per strip, tiles per strip
    int64_t NT;          // tiles
    uint64_t dir_off, streams_off;
};

__host__ __device__ inline uint64_t align16(uint64_t x) { return (x + 15) & ~uint64_t(15); }

__host__ __device__ inline Layout make_layout(int64_t N, int64_t K, int32_t B, int32_t vb)
{
    Layout L;
    L.N = N;
    L.K = K;
    L.B = B;
    L.vb = vb;
    L.S = 16 / B;
    L.KB = K / B;
    L.NS = (N + kStripRows - 1) / kStripRows;
    L.KP = (K + kPanelK - 1) / kPanelK;
    L.KT = (L.KP + kTilePanels - 1) / kTilePanels;
    L.NT = L.NS * L.KT;
    L.dir_off = kHeaderBytes;
    L.streams_off = align16(L.dir_off + uint64_t(L.NT + 1) * sizeof(DirEntry));
    return L;
}

__host__ __device__ inline int panels_in_tile(const Layout &L, int64_t kt)
{
    int64_t left = L.KP - kt * kTilePanels;
    return left < kTilePanels ? int(left) : kTilePanels;
}

// bytes of one tile's stream given its counts
__host__ __device__ inline uint32_t tile_bytes(const Layout &L, int npanels, uint32_t nU, uint32_t nD)
{
    (void)npanels;
    uint32_t b = uint32_t(kTilePanels) * 2u * uint32_t(L.S) * 8u;  // masks
    b += nU * uint32_t(L.vb);                                      // magnitudes
    b += (nU * uint32_t(L.B) + 7u) / 8u;                           // sign bits
    b = uint32_t(align16(b));                                      // dense blocks start 16-byte aligned
    b += nD * uint32_t(L.B) * uint32_t(L.vb);
    return uint32_t(align16(b));
}

// Position of element l's sign bit inside a block's B-bit sign field (see decode_block_bf16).
__host__ __device__ inline int sign_pos(int B, int l)
{
    switch (B) {
    case 16: return (l & 1) ? 15 - (l >> 1) : 7 - (l >> 1);
    case 8: return (l & 1) ? 3 - (l >> 1) : 7 - (l >> 1);
    case 4: return ((l & 1) << 1) | (((l >> 1) ^ 1) & 1);  // 0,1,2,3 -> 1,3,0,2
    default: return l;
    }
}

#if defined(__HIPCC__)

__device__ inline uint32_t mbcnt64(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi(uint32_t(m >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(m), 0u));
}

// Offsets of the three payload streams inside a tile stream.
struct TileStreams {
    uint32_t dense_off, mag_off, sign_off;
};

__device__ inline TileStreams tile_streams(int B, int vb, int npanels, uint32_t nU, uint32_t nD)
{
    TileStreams t;
    (void)npanels;
    (void)nD;
    t.mag_off = uint32_t(kTilePanels) * 2u * uint32_t(16 / B) * 8u;
    t.sign_off = t.mag_off + nU * uint32_t(vb);
    t.dense_off = (t.sign_off + (nU * uint32_t(B) + 7u) / 8u + 15u) & ~15u;
    return t;
}

// bf16 storage with B = 16 keeps {magnitude, sign field} of a UNIFIED block in one 32-bit record.
__host__ __device__ constexpr bool interleaved_records(int B, int vb) { return B == 16 && vb == 2; }

// The 32-bit record of a B = 16 bf16 UNIFIED block (q: 15 magnitude bits, field: sign_pos-permuted signs).
__host__ __device__ inline uint32_t pack_record16(uint32_t q, uint32_t field)
{
    return (q & 0xffu) | ((field & 0xffu) << 8) | ((q & 0xff00u) << 8) | ((field & 0xff00u) << 16);
}
__host__ __device__ inline void unpack_record16(uint32_t rec, uint32_t &q, uint32_t &field)
{
    q = (rec & 0xffu) | ((rec >> 8) & 0xff00u);
    field = ((rec >> 8) & 0xffu) | ((rec >> 16) & 0xff00u);
}

// Magnitude bits and B-bit sign field of the UNIFIED block with payload index `rank`.
// VB = value bytes (2: bf16 bits in the low half of q, 4: fp32 bits).
template <int B, int VB>
__device__ inline void load_unified(const uint8_t *tile, const TileStreams &ts, uint32_t rank, uint32_t &q,
                                    uint32_t &s)
{
    if constexpr (interleaved_records(B, VB)) {
        const uint32_t rec = reinterpret_cast<const uint32_t *>(tile + ts.mag_off)[rank];
        unpack_record16(rec, q, s);
    } else {
        if constexpr (VB == 2)
            q = reinterpret_cast<const uint16_t *>(tile + ts.mag_off)[rank];
        else
            q = reinterpret_cast<const uint32_t *>(tile + ts.mag_off)[rank];
        const uint8_t *signs = tile + ts.sign_off;
        if constexpr (B == 16) {
            s = reinterpret_cast<const uint16_t *>(signs)[rank];
        } else if constexpr (B == 8) {
            s = signs[rank];
        } else {
            const uint32_t bit = rank * B;
            s = (uint32_t(signs[bit >> 3]) >> (bit & 7u)) & ((1u << B) - 1u);
        }
    }
}

// One UNIFIED block -> B/2 dwords of bf16 pairs (element 2d in the low half of dword d).
// q has a clear sign bit, so each output dword is qq with bits 15 and 31 taken from the sign word:
// the encoder stores the signs so that ONE shift by d lines both bits up (sign_pos above).
template <int B>
__device__ inline void decode_block_bf16(uint32_t qbits, uint32_t sfield, uint32_t *out)
{
    const uint32_t qq = qbits | (qbits << 16);  // the stored magnitude is never negative: bit 15 is clear
    uint32_t sw;
    if constexpr (B == 16)
        sw = ((sfield & 0xffu) << 8) | ((sfield & 0xff00u) << 16);
    else if constexpr (B == 8)
        sw = (sfield << 8) | (sfield << 28);
    else if constexpr (B == 4)
        sw = (sfield << 14) | (sfield << 28);
    else
        sw = (sfield << 15) | (sfield << 30);
#pragma unroll
    for (int d = 0; d < B / 2; ++d) out[d] = qq | ((sw << d) & 0x80008000u);
}

#endif  // __HIPCC__

}  // namespace muw
