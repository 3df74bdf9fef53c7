// muw_stream.hip -- the memory-bound regime (M <= 16 activation rows, bf16): Y = X * W^^T where the
// time is the time to stream the compressed weights from HBM once (paper Sec. 3.2: the stored form of
// a pruned block is nothing, of a unified block one magnitude and B sign bits).
//
// The kernel is bound by vector-instruction issue (about one instruction per bf16 pair of decoded
// weights is the floor), so everything that is not decode runs on the scalar unit or not at all:
//   - persistent workgroups of 4 wavefronts, two per compute unit.  Wave w owns the quad of tile
//     columns 4 w .. 4 w + 3 (1024 consecutive k) and keeps the activations of those columns (all
//     M <= 16 rows: 128 registers of MFMA A-operands) for as long as the workgroup stays on one matrix;
//   - the quad's byte stream (4 tile streams, adjacent in the blob) goes HBM -> LDS with
//     global_load_lds_dwordx4 (no registers, no VALU) D strips ahead, into a per-wave ring of D + 1 slots;
//   - directory entries and the tile masks are fetched with scalar loads straight into scalar
//     registers (the masks one tile ahead; the lines are in L2 by then because the DMA asked for them
//     first), so masks cost no vector instruction; a lane finds its payload by v_mbcnt, reads it from
//     LDS (pruned blocks read nothing) and turns the record into bf16 pairs with one shift and one
//     bit-select per dword, straight into the B-operand of two 16x16x32 bf16 MFMAs per panel;
//   - the 4 partial 16x16 accumulators of a strip are summed through LDS by one wave (the role
//     rotates) and written to Y.  No atomics: results are bitwise reproducible.
// Every quad issues exactly NCHS 1-KiB DMA instructions (lanes past the end of the stream re-read its
// last 16 bytes) and every iteration one more for a directory span, so "strip q has landed" is a static
// vmcnt wait.  Inside a quad everything follows from the tile masks (record and dense offsets, the
// tile's size, hence the next tile's address): the directory is needed only for the quad's span.
#include "muw_decode.hpp"
#include "muw_internal.hpp"

namespace muw {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;
// Explicit address spaces: a pointer read from a device pointer table is "generic" to the compiler,
// and generic (flat) accesses count in both memory counters and force full drains.
typedef __attribute__((address_space(1))) const u32x4_t g_cu32x4;
typedef __attribute__((address_space(1))) const uint32_t g_cu32;
typedef __attribute__((address_space(1))) float g_float;
typedef __attribute__((address_space(1))) uint16_t g_u16;
typedef const __attribute__((address_space(4))) uint64_t c_u64;

constexpr int kWaves = 4;                   // wavefronts per workgroup
constexpr int kCols = 4;                    // tile columns per wavefront (a "quad": contiguous in the blob)
constexpr int kChunkCols = kWaves * kCols;  // tile columns per workgroup (4096 k); more K goes to blockIdx.y
constexpr int kP = kTilePanels;             // panels per tile (4)
static_assert(kP == 4, "the streaming kernel is written for 4-panel tiles");
typedef const __attribute__((address_space(4))) uint32_t c_u32;

struct StreamArgs {
    const uint8_t *blob;
    const uint16_t *X;
    void *Y;
    const void *const *blobs;  // grouped: device arrays of G pointers (else null)
    const void *const *Xs;
    void *const *Ys;
    int32_t G, M;
    int32_t ldx, ldy;  // row strides in elements (M <= 16 rows: 32-bit offsets suffice)
    int32_t ydtype;
    int32_t nstrips;  // G * NS: strips over all matrices
    int32_t per_wg;   // strips per workgroup
    float *Ypart;     // [nchunk][G][M][N] partial sums when K is split over blockIdx.y, else null
    int32_t nchunk;
};

// The few layout numbers the kernel needs (32-bit, to keep scalar registers free).
struct StreamGeom {
    uint32_t dir_off, streams_off;
    int32_t KT, NS, N, K;
};

// Entry i of a device table of pointers, through the scalar cache (i is wave-uniform).
__device__ inline uint64_t table_entry(const void *table, int i) { return ((c_u64 *)table)[i]; }

// Workgroup barrier for LDS traffic only: waits for this wave's LDS operations, not for the DMA
// prefetches in flight (a full __syncthreads() drains vmcnt as well).
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int N>
__device__ inline void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    // gfx9 s_waitcnt: vmcnt = simm16[15:14]:[3:0], expcnt = [6:4], lgkmcnt = [11:8] (left untouched)
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}

// LDS reads of DMA-filled memory are written as inline assembly on purpose: for an ordinary LDS
// load that may alias a pending global_load_lds the compiler inserts a wait for ALL pending DMA,
// which would cancel the prefetch distance.  Here the slot discipline (a slot is read only after the
// explicit vmcnt wait for its own DMA, and refilled only after its last read has returned) is the
// proof of ordering, and every batch of reads is followed by one explicit lgkmcnt(0) whose operands
// tie it to the registers it guards.
__device__ inline uint32_t lds_offset(const void *p)
{
    return uint32_t(reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) uint8_t *)p));
}
__device__ inline uint32_t lds_read_b32(uint32_t addr)
{
    uint32_t dst;
    asm volatile("ds_read_b32 %0, %1" : "=v"(dst) : "v"(addr));
    return dst;
}
__device__ inline uint32_t lds_read_u16(uint32_t addr)
{
    uint32_t dst;
    asm volatile("ds_read_u16 %0, %1" : "=v"(dst) : "v"(addr));
    return dst;
}
__device__ inline uint32_t lds_read_u8(uint32_t addr)
{
    uint32_t dst;
    asm volatile("ds_read_u8 %0, %1" : "=v"(dst) : "v"(addr));
    return dst;
}
__device__ inline void lds_read_2xb128(u32x4_t &lo, u32x4_t &hi, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:16" : "=&v"(lo), "=&v"(hi) : "v"(addr));
}
__device__ inline u32x4_t lds_read_b128(uint32_t addr)
{
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}
__device__ inline uint64_t lds_read_b64(uint32_t addr)
{
    uint64_t v;
    asm volatile("ds_read_b64 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}

__device__ inline uint64_t uniform64(uint64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(v >> 32));
    return (uint64_t(hi) << 32) | lo;
}

// ------------------------------------------------------------------------------------------------
// B = 16: the tile's 8 masks (4 panels x {U, D}) are the first 64 bytes of its stream.
// ------------------------------------------------------------------------------------------------
struct TileMasks16 {
    uint64_t u[kP], d[kP];
};

// Scalar load of a tile's masks from the blob (address is wave-uniform).
__device__ inline void load_masks16(TileMasks16 &m, uint64_t tile_addr)
{
    c_u64 *p = (c_u64 *)tile_addr;
#pragma unroll
    for (int i = 0; i < kP; ++i) {
        m.u[i] = p[2 * i];
        m.d[i] = p[2 * i + 1];
    }
}

// Bytes of a B = 16 bf16 tile stream, from its masks: 64 (masks) + 4 per UNIFIED block, rounded up to
// 16, + 32 per DENSE block.  `dense_rel` = offset of the first DENSE block.
__device__ inline uint32_t tile_bytes16(const TileMasks16 &m, uint32_t &dense_rel)
{
    uint32_t nU = 0, nD = 0;
#pragma unroll
    for (int p = 0; p < kP; ++p) {
        nU += uint32_t(__popcll(m.u[p]));
        nD += uint32_t(__popcll(m.d[p]));
    }
    dense_rel = kP * 16u + ((nU * 4u + 15u) & ~15u);
    return dense_rel + nD * 32u;
}

// One tile (4 panels) of a B = 16 layer: issue every payload read, wait once, run `mid` (scalar and
// DMA work that should overlap the decode), decode, 8 MFMAs.
// Record layout (pack_record16): bytes {q low, signs of even elements, q high, signs of odd elements},
// so (rec << d) has the signs of elements 2 d and 2 d + 1 at bits 15 and 31.
template <int T, typename Mid>
__device__ inline void process_tile16(uint32_t tile_lds, uint32_t dense_rel, const TileMasks16 &m,
                                      const uint4 (&xr)[kCols * kP][2], f32x4 &acc0, f32x4 &acc1, uint64_t &extra,
                                      Mid mid)
{
    uint32_t s_rec = tile_lds + kP * 16u;      // scalar: running LDS address of the next record
    uint32_t s_dense = tile_lds + dense_rel;   // scalar: running LDS address of the next DENSE block
    uint32_t rec[kP];
    u32x4_t wlo[kP], whi[kP];
#pragma unroll
    for (int p = 0; p < kP; ++p) {
        // Every lane reads (a lane without a UNIFIED block reads a neighbour's record and drops it
        // below): an unconditional read leaves no register copy between the read and the wait.
        rec[p] = lds_read_b32(s_rec + 4u * mbcnt64(m.u[p]));
        if (__builtin_amdgcn_inverse_ballot_w64(m.d[p])) lds_read_2xb128(wlo[p], whi[p], s_dense + 32u * mbcnt64(m.d[p]));
        s_rec += 4u * uint32_t(__popcll(m.u[p]));
        s_dense += 32u * uint32_t(__popcll(m.d[p]));
    }
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(rec[0]), "+v"(rec[1]), "+v"(rec[2]), "+v"(rec[3]), "+v"(wlo[0]), "+v"(wlo[1]),
                   "+v"(wlo[2]), "+v"(wlo[3]), "+v"(whi[0]), "+v"(whi[1]), "+v"(whi[2]), "+v"(whi[3]), "+v"(extra));
    mid();
#pragma unroll
    for (int p = 0; p < kP; ++p) {
        if (!__builtin_amdgcn_inverse_ballot_w64(m.d[p])) {
            const uint32_t rc = __builtin_amdgcn_inverse_ballot_w64(m.u[p]) ? rec[p] : 0u;
            const uint32_t qq = __builtin_amdgcn_perm(rc, rc, 0x02000200u);
            wlo[p].x = qq | (rc & 0x80008000u);
            wlo[p].y = qq | ((rc << 1) & 0x80008000u);
            wlo[p].z = qq | ((rc << 2) & 0x80008000u);
            wlo[p].w = qq | ((rc << 3) & 0x80008000u);
            whi[p].x = qq | ((rc << 4) & 0x80008000u);
            whi[p].y = qq | ((rc << 5) & 0x80008000u);
            whi[p].z = qq | ((rc << 6) & 0x80008000u);
            whi[p].w = qq | ((rc << 7) & 0x80008000u);
        }
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xr[T * kP + p][0]),
                                                       __builtin_bit_cast(bf16x8, wlo[p]), acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xr[T * kP + p][1]),
                                                       __builtin_bit_cast(bf16x8, whi[p]), acc1, 0, 0, 0);
    }
}

// ------------------------------------------------------------------------------------------------
// B = 4, 8: same walk, panel by panel, masks read from the LDS copy when needed (not tuned: these
// block lengths are not on the memory-bound benchmark).
// ------------------------------------------------------------------------------------------------
// Block counts of a tile from its masks in the blob (scalar loads).
template <int B>
__device__ inline void tile_counts_small_b(uint64_t tile_addr, uint32_t &nU, uint32_t &nD)
{
    constexpr int S = 16 / B;
    c_u64 *p = (c_u64 *)tile_addr;
    nU = nD = 0;
#pragma unroll 1
    for (int pn = 0; pn < kP; ++pn)
#pragma unroll
        for (int jj = 0; jj < S; ++jj) {
            nU += uint32_t(__popcll(p[pn * 2 * S + jj]));
            nD += uint32_t(__popcll(p[pn * 2 * S + S + jj]));
        }
}

template <int B, int T>
__device__ inline uint32_t process_tile_small_b(uint32_t tile_lds, uint32_t nU, uint32_t nD,
                                                const uint4 (&xr)[kCols * kP][2], f32x4 &acc0, f32x4 &acc1)
{
    constexpr int S = 16 / B;
    constexpr uint32_t mag_off = kP * 2u * S * 8u;
    const uint32_t sign_off = mag_off + nU * 2u;
    const uint32_t dense_off = (sign_off + (nU * uint32_t(B) + 7u) / 8u + 15u) & ~15u;
    uint32_t ru = 0, rd = 0;
#pragma unroll
    for (int p = 0; p < kP; ++p) {
        uint32_t w[8];
#pragma unroll
        for (int j = 0; j < S; ++j) {
            uint64_t mu_v = lds_read_b64(tile_lds + uint32_t(p * 2 * S + j) * 8u);
            uint64_t md_v = lds_read_b64(tile_lds + uint32_t(p * 2 * S + S + j) * 8u);
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(mu_v), "+v"(md_v));
            const uint64_t mu = uniform64(mu_v), md = uniform64(md_v);
            const uint32_t rku = ru + mbcnt64(mu), rkd = rd + mbcnt64(md);
            ru += __popcll(mu);
            rd += __popcll(md);
            uint32_t q = lds_read_u16(tile_lds + mag_off + 2u * rku);
            const uint32_t bit = rku * B;
            uint32_t s = lds_read_u8(tile_lds + sign_off + (bit >> 3));
            u32x4_t dn = {0, 0, 0, 0};
            if (__builtin_amdgcn_inverse_ballot_w64(md)) {
                if constexpr (B == 8) {
                    dn = lds_read_b128(tile_lds + dense_off + 16u * rkd);
                } else {
                    const uint64_t t = lds_read_b64(tile_lds + dense_off + 8u * rkd);
                    dn.x = uint32_t(t);
                    dn.y = uint32_t(t >> 32);
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(q), "+v"(s), "+v"(dn));
            s = (s >> (bit & 7u)) & ((1u << B) - 1u);
            if (!__builtin_amdgcn_inverse_ballot_w64(mu)) {
                q = 0;
                s = 0;
            }
            decode_block_bf16<B>(q, s, w + j * (B / 2));
            if (__builtin_amdgcn_inverse_ballot_w64(md)) {
                w[j * (B / 2)] = dn.x;
                w[j * (B / 2) + 1] = dn.y;
                if constexpr (B == 8) {
                    w[j * (B / 2) + 2] = dn.z;
                    w[j * (B / 2) + 3] = dn.w;
                }
            }
        }
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, xr[T * kP + p][0]), __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3])),
            acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, xr[T * kP + p][1]), __builtin_bit_cast(bf16x8, make_uint4(w[4], w[5], w[6], w[7])),
            acc1, 0, 0, 0);
    }
    return (dense_off + nD * uint32_t(B) * 2u + 15u) & ~15u;  // bytes of this tile stream
}

// Where a workgroup is in its sequence of strips (which runs over all matrices of a grouped call).
struct Cursor {
    int32_t gi, strip;
    uint64_t blob;
};

struct StreamKernArgs {
    StreamArgs a;
    StreamGeom L;
};
// A kernel argument read where it is used (through the scalar cache) instead of being kept in a
// scalar register for the whole kernel: the loop needs those registers for the tile masks.
template <typename T>
__device__ inline T kernarg(size_t offset)
{
    const __attribute__((address_space(4))) uint8_t *p =
        (const __attribute__((address_space(4))) uint8_t *)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(p));  // opaque: keeps the load from being hoisted out of the loop
    return *(const __attribute__((address_space(4))) T *)(p + offset);
}
#define MUW_KARG(type, field) kernarg<type>(offsetof(StreamKernArgs, field))

// SLOT512: bytes of a ring slot in units of 512 (>= the largest quad of the blob).
template <int B, int SLOT512, int D>
__global__ __launch_bounds__(kWaves * 64, 2) void k_stream_bf16(StreamKernArgs)
{
    constexpr int SLOT = SLOT512 * 512;
    constexpr int NCHS = (SLOT + 1023) / 1024;  // DMA instructions per quad
    constexpr int NSLOT = D + 1;
    constexpr int NSPAN = 2 * D + 1;
    constexpr int PER_ITER = NCHS + 1;  // DMA instructions per steady-state iteration (span + quad)
    __shared__ __attribute__((aligned(16))) uint8_t ring[kWaves][NSLOT * SLOT];
    __shared__ __attribute__((aligned(16))) float red[2][kWaves][64][4];
    // {first, one-past-last} stream offset of the wave's quad in upcoming strips (fetched by DMA far
    // ahead: a scalar load of a cold directory line would stall every wait on the scalar/LDS counter)
    __shared__ __attribute__((aligned(8))) uint32_t spans[kWaves][NSPAN][2];

    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    const int kt0 = int(blockIdx.y) * kChunkCols + wave * kCols;
    // the few arguments the loop needs all the time
    const uint32_t KT = MUW_KARG(int32_t, L.KT), NS = MUW_KARG(int32_t, L.NS);
    const uint32_t dir_off = MUW_KARG(uint32_t, L.dir_off), streams_off = MUW_KARG(uint32_t, L.streams_off);
    const int ncols = int(KT) - kt0 < kCols ? int(KT) - kt0 : kCols;  // tile columns this wave has (<= 0: none)
    const bool active = ncols > 0;

    int nseq;   // this workgroup's strips, over all matrices: element q = strip s_lo + q
    Cursor cc;  // strip being decoded
    {
        const int per_wg = MUW_KARG(int32_t, a.per_wg), nstrips = MUW_KARG(int32_t, a.nstrips);
        const int s_lo = blockIdx.x * per_wg;
        int s_hi = s_lo + per_wg;
        if (s_hi > nstrips) s_hi = nstrips;
        if (s_lo >= s_hi) return;
        nseq = s_hi - s_lo;
        cc.gi = s_lo / int(NS);
        cc.strip = s_lo % int(NS);
    }
    const uint32_t myring = lds_offset(ring[wave]);

    auto blob_of = [&](int gi) -> uint64_t {
        const void *const *blobs = MUW_KARG(const void *const *, a.blobs);
        return blobs ? table_entry(blobs, gi) : reinterpret_cast<uint64_t>(MUW_KARG(const uint8_t *, a.blob));
    };
    auto advance = [&](Cursor &c) {  // (callers never step past the last strip of the last matrix)
        if (++c.strip == int(NS)) {
            c.strip = 0;
            ++c.gi;
            c.blob = blob_of(c.gi);
        }
    };
    // ---- DMA of the span {first, one-past-last offset} of the wave's quad in strip c: lanes 0 and 1
    //      fetch one directory word each
    auto issue_span = [&](const Cursor &c, int sslot) {
        const uint64_t e = c.blob + dir_off + uint64_t(uint32_t(c.strip) * KT + uint32_t(kt0)) * sizeof(DirEntry);
        if (lane < 2)
            __builtin_amdgcn_global_load_lds((global_void_t *)(e + (lane ? uint32_t(ncols) * 8u : 0u)),
                                             (lds_void_t *)spans[wave][sslot], 4, 0, 0);
    };
    // ---- the NCHS DMA instructions of one quad into ring slot `slot`
    auto issue_quad = [&](int slot, uint64_t base, uint32_t bytes) {
        const uint32_t last = bytes - 16u;
#pragma unroll
        for (int c = 0; c < NCHS; ++c) {
            uint32_t off = uint32_t(c) * 1024u + uint32_t(lane) * 16u;
            off = off < last ? off : last;
            if (c * 1024 + 1024 <= SLOT || lane < 32)  // (a slot may end in the middle of the last KiB)
                __builtin_amdgcn_global_load_lds((global_void_t *)(base + off),
                                                 (lds_void_t *)(ring[wave] + slot * SLOT + c * 1024), 16, 0, 0);
        }
    };
    auto next_slot = [](int sl, int n) { return sl + 1 == n ? 0 : sl + 1; };

    uint4 xr[kCols * kP][2];
#pragma unroll
    for (int p = 0; p < kCols * kP; ++p) xr[p][0] = xr[p][1] = make_uint4(0, 0, 0, 0);
    int cur_g = -1;

    cc.blob = blob_of(cc.gi);
    Cursor cq = cc;            // strip whose quad DMA is issued next (q + D in the loop)
    Cursor cs = cc;            // strip whose span DMA is issued next (q + 2 D in the loop)
    int n_cs = 0;              // its index in the sequence (stops at nseq - 1: then the last span is re-fetched)
    uint64_t tg = 0;           // address in the blob of the tile decoded next
    uint64_t fifo[D] = {};     // addresses of the quads of strips q + 1 .. q + D
    TileMasks16 mk{};          // B = 16: masks of the tile decoded next
    int slot_issue = 0, slot_proc = 0, span_issue = 0, span_read = 0;

    auto step_span_cursor = [&]() {
        if (n_cs + 1 < nseq) {
            ++n_cs;
            advance(cs);
        }
    };
    // the quad of the strip at cursor cq: read its span (landed), issue its DMA, return its address
    auto start_quad = [&](uint64_t span) -> uint64_t {
        const uint32_t begin = __builtin_amdgcn_readfirstlane(uint32_t(span));
        const uint32_t end = __builtin_amdgcn_readfirstlane(uint32_t(span >> 32));
        const uint64_t base = cq.blob + streams_off + uint64_t(begin) * 16u;
        issue_quad(slot_issue, base, (end - begin) * 16u);
        slot_issue = next_slot(slot_issue, NSLOT);
        return base;
    };

    if (active) {
        // spans of strips 0 .. D - 1, then (as iterations -D .. -1 of the loop would) span j + 2 D and quad j + D
        for (int i = 0; i < D; ++i) {
            issue_span(cs, span_issue);
            span_issue = next_slot(span_issue, NSPAN);
            step_span_cursor();
        }
        wait_vmcnt<0>();
        for (int i = 0; i < D; ++i) {
            issue_span(cs, span_issue);
            span_issue = next_slot(span_issue, NSPAN);
            step_span_cursor();
            uint64_t span = lds_read_b64(lds_offset(spans[wave][span_read]));
            span_read = next_slot(span_read, NSPAN);
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(span));
            if (i < nseq) {
                const uint64_t base = start_quad(span);
                if (i == 0)
                    tg = base;
                else
                    fifo[i - 1] = base;
                if (i + 1 < nseq) advance(cq);
            }
        }
        if constexpr (B == 16) load_masks16(mk, tg);
    }

    for (int q = 0; q < nseq; ++q) {
        if (cc.gi != cur_g) {
            cur_g = cc.gi;
            if (active) {
                const void *const *Xs = MUW_KARG(const void *const *, a.Xs);
                const uint64_t X = Xs ? table_entry(Xs, cc.gi) : reinterpret_cast<uint64_t>(MUW_KARG(const uint16_t *, a.X));
                const int ldx = MUW_KARG(int32_t, a.ldx), M = MUW_KARG(int32_t, a.M), K = MUW_KARG(int32_t, L.K);
                const int r = lane & 15, g4 = lane >> 4;
#pragma unroll
                for (int p = 0; p < kCols * kP; ++p)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int k = kt0 * kTileK + p * kPanelK + 16 * g4 + 8 * h;
                        uint4 v = make_uint4(0, 0, 0, 0);
                        if (r < M && k + 8 <= K) {
                            const u32x4_t t = *(g_cu32x4 *)(X + uint64_t(uint32_t(r * ldx + k) * 2u));
                            v = make_uint4(t.x, t.y, t.z, t.w);
                        }
                        xr[p][h] = v;
                    }
                // Drain here, once per matrix, so that no later use of xr needs a wait that would also
                // wait for the DMA prefetches in flight.
                wait_vmcnt<0>();
            }
        }
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        Cursor cn = cc;  // strip q + 1 (every wave steps: the reducing wave needs it even without tile columns)
        if (q + 1 < nseq) advance(cn);
        if (active) {
            // Quad q has landed, and so has the span of strip q + D: everything but the DMA of the last
            // D - 1 iterations (which all issued a span and a quad if strip q + D - 1 exists).
            if (q + D <= nseq)
                wait_vmcnt<(D - 1) * PER_ITER>();
            else
                wait_vmcnt<0>();
            uint64_t span = lds_read_b64(lds_offset(spans[wave][span_read]));  // waited for inside tile 0
            span_read = next_slot(span_read, NSPAN);
            // after the payload wait of tile 0: DMA for strip q + D (its span is in registers now) and
            // the span of strip q + 2 D
            auto start_dma = [&]() {
                issue_span(cs, span_issue);
                span_issue = next_slot(span_issue, NSPAN);
                step_span_cursor();
                if (q + D < nseq) {
                    fifo[D - 1] = start_quad(span);
                    if (q + D + 1 < nseq) advance(cq);
                }
            };
            uint32_t tl = myring + uint32_t(slot_proc) * SLOT;
            slot_proc = next_slot(slot_proc, NSLOT);
            uint64_t unused = 0;
#pragma unroll
            for (int t = 0; t < kCols; ++t) {
                if (t < ncols) {
                    // the tile decoded after this one: next in the quad, else first of the next strip's
                    // quad (after the very last tile: this one again, unused)
                    const bool last_tile = t + 1 >= ncols;
                    if constexpr (B == 16) {
                        uint32_t dense_rel;
                        const uint32_t tbytes = tile_bytes16(mk, dense_rel);
                        uint64_t tg_next = tg + tbytes;
                        if (last_tile) tg_next = q + 1 < nseq ? fifo[0] : tg;
                        TileMasks16 mnext;
                        auto mid = [&]() {
                            if (t == 0) start_dma();
                            // (opaque: the scalar load must not move above the wait it follows, or that
                            // wait would include its latency)
                            uint64_t addr = last_tile && t == 0 && q + 1 < nseq ? fifo[0] : tg_next;
                            asm volatile("" : "+s"(addr));
                            load_masks16(mnext, addr);
                        };
                        if (t == 0) process_tile16<0>(tl, dense_rel, mk, xr, acc0, acc1, span, mid);
                        if (t == 1) process_tile16<1>(tl, dense_rel, mk, xr, acc0, acc1, unused, mid);
                        if (t == 2) process_tile16<2>(tl, dense_rel, mk, xr, acc0, acc1, unused, mid);
                        if (t == 3) process_tile16<3>(tl, dense_rel, mk, xr, acc0, acc1, unused, mid);
                        mk = mnext;
                        tg = tg_next;
                        tl += tbytes;
                    } else {
                        if (t == 0) {
                            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(span));
                            start_dma();
                        }
                        uint32_t nU, nD, tbytes = 0;
                        tile_counts_small_b<B>(tg, nU, nD);
                        if (t == 0) tbytes = process_tile_small_b<B, 0>(tl, nU, nD, xr, acc0, acc1);
                        if (t == 1) tbytes = process_tile_small_b<B, 1>(tl, nU, nD, xr, acc0, acc1);
                        if (t == 2) tbytes = process_tile_small_b<B, 2>(tl, nU, nD, xr, acc0, acc1);
                        if (t == 3) tbytes = process_tile_small_b<B, 3>(tl, nU, nD, xr, acc0, acc1);
                        tg += tbytes;
                        if (last_tile && q + 1 < nseq) tg = fifo[0];
                        tl += tbytes;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i + 1 < D; ++i) fifo[i] = fifo[i + 1];
        }
        *reinterpret_cast<f32x4 *>(red[q & 1][wave][lane]) = acc0 + acc1;
        lds_barrier();
        if (wave == (q & (kWaves - 1))) {
            // (asm reads for the same reason as the tile reads: no wait on the DMA in flight)
            f32x4 part[kWaves];
#pragma unroll
            for (int w2 = 0; w2 < kWaves; ++w2)
                asm volatile("ds_read_b128 %0, %1" : "=v"(part[w2]) : "v"(lds_offset(red[q & 1][w2][lane])));
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(part[0]), "+v"(part[1]), "+v"(part[2]), "+v"(part[3]));
            const f32x4 t = (part[0] + part[1]) + (part[2] + part[3]);  // waves without a tile column wrote zeros
            const int r = lane & 15, g4 = lane >> 4;
            const int n = cc.strip * kStripRows + r;
            const int N = MUW_KARG(int32_t, L.N), M = MUW_KARG(int32_t, a.M);
            float *Ypart = MUW_KARG(float *, a.Ypart);
            if (n < N) {
                if (Ypart) {
                    const int G = MUW_KARG(int32_t, a.G);
                    const uint64_t Yp = reinterpret_cast<uint64_t>(Ypart) +
                                        uint64_t(int64_t(blockIdx.y) * G + cc.gi) * uint64_t(M) * uint64_t(N) * 4u;
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (4 * g4 + v < M) *(g_float *)(Yp + uint64_t(uint32_t((4 * g4 + v) * N + n) * 4u)) = t[v];
                } else {
                    void *const *Ys = MUW_KARG(void *const *, a.Ys);
                    const uint64_t Y = Ys ? table_entry(Ys, cc.gi) : reinterpret_cast<uint64_t>(MUW_KARG(void *, a.Y));
                    const int ldy = MUW_KARG(int32_t, a.ldy);
                    const bool f32out = MUW_KARG(int32_t, a.ydtype) == MUW_F32;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int m = 4 * g4 + v;
                        if (m >= M) continue;
                        if (f32out)
                            *(g_float *)(Y + uint64_t(uint32_t(m * ldy + n) * 4u)) = t[v];
                        else
                            *(g_u16 *)(Y + uint64_t(uint32_t(m * ldy + n) * 2u)) = f32_to_bf16_rne(t[v]);
                    }
                }
            }
        }
        cc = cn;
    }
}

// Sum the K-chunk partials (in chunk order: deterministic) and write Y.
__global__ __launch_bounds__(256) void k_stream_reduce(const float *Ypart, int nchunk, int G, int M,
                                                       int64_t N, void *Y, void *const *Ys, int64_t ldy,
                                                       int ydtype)
{
    const int64_t per = int64_t(M) * N;
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= per * G) return;
    const int64_t gi = i / per, rem = i % per, m = rem / N, n = rem % N;
    float t = 0.f;
    for (int c = 0; c < nchunk; ++c) t += Ypart[(int64_t(c) * G + gi) * per + rem];
    void *out = Ys ? Ys[gi] : Y;
    if (ydtype == MUW_F32)
        static_cast<float *>(out)[m * ldy + n] = t;
    else
        static_cast<uint16_t *>(out)[m * ldy + n] = f32_to_bf16_rne(t);
}

int device_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

template <int B, int SLOT512, int D>
muw_status launch_stream_variant(StreamArgs a, const Layout &L, hipStream_t st)
{
    const StreamGeom geom{uint32_t(L.dir_off), uint32_t(L.streams_off), int32_t(L.KT), int32_t(L.NS),
                          int32_t(L.N), int32_t(L.K)};
    const int wgs = 2 * device_cus();  // two workgroups per compute unit
    a.nstrips = int32_t(L.NS) * a.G;
    int grid = a.nstrips < wgs ? a.nstrips : wgs;
    a.per_wg = (a.nstrips + grid - 1) / grid;
    grid = (a.nstrips + a.per_wg - 1) / a.per_wg;
    dim3 g(unsigned(grid), unsigned(a.nchunk), 1);
    k_stream_bf16<B, SLOT512, D><<<g, kWaves * 64, 0, st>>>(StreamKernArgs{a, geom});
    return hip_status(hipGetLastError());
}

template <int B>
muw_status launch_stream_b(StreamArgs a, const Layout &L, int quad_bytes, hipStream_t st)
{
    // Per-wave ring of (D + 1) slots that hold one quad each; two workgroups (4 rings + reduction
    // buffers each) share the 160 KiB of LDS of a compute unit while a slot is at most 5.5 KiB.
    const int slot512 = (quad_bytes + 511) / 512;
    if (slot512 <= 8) return launch_stream_variant<B, 8, 2>(a, L, st);
    if (slot512 <= 10) return launch_stream_variant<B, 10, 2>(a, L, st);
    if (slot512 <= 11) return launch_stream_variant<B, 11, 2>(a, L, st);
    if (slot512 <= 12) return launch_stream_variant<B, 12, 2>(a, L, st);
    if (slot512 <= 16) return launch_stream_variant<B, 16, 2>(a, L, st);
    return MUW_EUNSUPPORTED;
}

}  // namespace

// Can the streaming kernel take this problem?  (bf16, M <= 16, 16-byte aligned activation rows, tile
// streams that fit the LDS ring.)
bool stream_gemm_applicable(const muw_desc &d, const Layout &L, const GemmArgs &a)
{
    if (d.wdtype != MUW_BF16 || a.M > 16 || a.M < 1) return false;
    if (d.max_quad_bytes <= 0 || d.max_quad_bytes > 8192) return false;
    if (L.K % 8 != 0 || a.ldx % 8 != 0) return false;
    if (a.ldx >= (1 << 26) || a.ldy >= (1 << 26) || L.N >= (1 << 26)) return false;  // 32-bit offsets in the kernel
    if (!a.blobs && (reinterpret_cast<uintptr_t>(a.X) & 15u)) return false;
    if (a.G > 32767 || L.NS * int64_t(a.G) > (int64_t(1) << 30) || L.NT >= (int64_t(1) << 28)) return false;
    return true;
}

size_t stream_gemm_workspace_bytes(const Layout &L, int64_t M, int G)
{
    const int64_t nchunk = (L.KT + kChunkCols - 1) / kChunkCols;
    return nchunk > 1 ? size_t(nchunk) * size_t(G) * size_t(M) * size_t(L.N) * sizeof(float) : 0;
}

muw_status launch_stream_gemm(const muw_desc &d, const Layout &L, const GemmArgs &g, void *ws, hipStream_t st)
{
    StreamArgs a{};
    a.blob = static_cast<const uint8_t *>(g.blob);
    a.X = static_cast<const uint16_t *>(g.X);
    a.Y = g.Y;
    a.blobs = g.blobs;
    a.Xs = g.Xs;
    a.Ys = g.Ys;
    a.G = g.blobs ? g.G : 1;
    a.M = int32_t(g.M);
    a.ldx = int32_t(g.ldx);
    a.ldy = int32_t(g.ldy);
    a.ydtype = g.ydtype;
    a.nchunk = int32_t((L.KT + kChunkCols - 1) / kChunkCols);
    a.Ypart = a.nchunk > 1 ? static_cast<float *>(ws) : nullptr;
    muw_status rc;
    switch (d.B) {
    case 4: rc = launch_stream_b<4>(a, L, d.max_quad_bytes, st); break;
    case 8: rc = launch_stream_b<8>(a, L, d.max_quad_bytes, st); break;
    case 16: rc = launch_stream_b<16>(a, L, d.max_quad_bytes, st); break;
    default: return MUW_EUNSUPPORTED;
    }
    if (rc != MUW_OK) return rc;
    if (a.nchunk > 1) {
        const int64_t total = int64_t(a.G) * a.M * L.N;
        k_stream_reduce<<<unsigned((total + 255) / 256), 256, 0, st>>>(a.Ypart, a.nchunk, a.G, a.M, L.N, g.Y,
                                                                      g.Ys, g.ldy, g.ydtype);
        rc = hip_status(hipGetLastError());
    }
    return rc;
}

}  // namespace muw
