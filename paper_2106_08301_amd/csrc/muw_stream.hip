// muw_stream.hip -- the memory-bound regime (M <= 16 activation rows, bf16): Y = X * W^^T where the
// time is the time to stream the compressed weights from HBM once (paper Sec. 3.2: the stored form of
// a pruned block is nothing, of a unified block one magnitude and B sign bits).
//
// One persistent workgroup of 8 wavefronts per compute unit.  Wave w keeps the activations of tile
// column kt = 8 c + w (512 consecutive k, all M <= 16 rows) in registers as MFMA A-operands for as
// long as the workgroup stays on one weight matrix, and walks down the strips (16 output rows) of
// that tile column:
//   - the tile's byte stream goes HBM -> LDS with global_load_lds_dwordx4 (no registers, no VALU),
//     D tiles ahead of the one being decoded, into a per-wave ring of D+1 slots;
//   - the lane decodes its 16 weights of each panel from LDS (mask -> payload index by v_mbcnt,
//     magnitude | sign bits -> bf16 pairs with one shift and one bit-select per dword; pruned blocks
//     read no payload) straight into the B-operand of two 16x16x32 bf16 MFMAs;
//   - after SPI strips the 8 partial 16x16 accumulators of a strip (one per tile column) are summed
//     through LDS by one wave (the role rotates) and written to Y.  No atomics: results are
//     bitwise reproducible.
// Every tile issues exactly NCH 1-KiB DMA instructions (lanes past the end of the stream re-read its
// last 16 bytes), so "tile q has landed" is the static wait vmcnt(D * NCH).
#include "muw_decode.hpp"
#include "muw_internal.hpp"

namespace muw {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

struct StreamArgs {
    const uint8_t *blob;
    const uint16_t *X;
    void *Y;
    const void *const *blobs;  // grouped: device arrays of G pointers (else null)
    const void *const *Xs;
    void *const *Ys;
    int32_t G, M;
    int64_t ldx, ldy;
    int32_t ydtype;
    int32_t nbpm;      // batches (of SPI strips) per matrix
    int32_t nbatches;  // G * nbpm
    int32_t per_wg;    // batches per workgroup
    float *Ypart;      // [nchunk][G][M][N] partial sums when K is split over blockIdx.y, else null
    int32_t nchunk;
};

// Explicit address spaces: a pointer read from a device pointer table is "generic" to the compiler,
// and generic (flat) accesses count in both memory counters and force full drains.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const u32x4_t g_cu32x4;
typedef __attribute__((address_space(1))) const uint32_t g_cu32;
typedef __attribute__((address_space(1))) float g_float;
typedef __attribute__((address_space(1))) uint16_t g_u16;
typedef const __attribute__((address_space(4))) uint64_t c_u64;

// Entry i of a device table of pointers, through the scalar cache (i is wave-uniform).
__device__ inline uint64_t table_entry(const void *table, int i) { return ((c_u64 *)table)[i]; }

// Workgroup barrier for LDS traffic only: waits for this wave's LDS operations, not for the DMA
// prefetches in flight (a full __syncthreads() drains vmcnt as well).
__device__ inline void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int N>
__device__ inline void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    // gfx9 s_waitcnt: vmcnt = simm16[15:14]:[3:0], expcnt = [6:4], lgkmcnt = [11:8] (left untouched)
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}

__device__ inline uint64_t uniform64(uint64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(v >> 32));
    return (uint64_t(hi) << 32) | lo;
}

// ---- B < 16: masks are read from the LDS copy of the tile and made wave-uniform ------------------
template <int B>
__device__ inline void decode_panel_lds(const uint8_t *tile, const TileStreams &ts, int p, uint32_t &ru,
                                        uint32_t &rd, uint32_t *w)
{
    constexpr int S = 16 / B;
    const uint64_t *masks = reinterpret_cast<const uint64_t *>(tile) + p * 2 * S;
#pragma unroll
    for (int j = 0; j < S; ++j) {
        const uint64_t mu = uniform64(masks[j]), md = uniform64(masks[S + j]);
        const uint32_t rku = ru + mbcnt64(mu), rkd = rd + mbcnt64(md);
        ru += __popcll(mu);
        rd += __popcll(md);
        uint32_t q = 0, s = 0;
        if (__builtin_amdgcn_inverse_ballot_w64(mu)) load_unified<B, 2>(tile, ts, rku, q, s);
        decode_block_bf16<B>(q, s, w + j * (B / 2));
        if (__builtin_amdgcn_inverse_ballot_w64(md)) {
            const uint32_t *src = reinterpret_cast<const uint32_t *>(tile + ts.dense_off) + rkd * (B / 2);
#pragma unroll
            for (int d = 0; d < B / 2; ++d) w[j * (B / 2) + d] = src[d];
        }
    }
}

template <int B>
__device__ inline void process_tile_generic(const uint8_t *tile, int np, int npq, uint32_t nU, uint32_t nD,
                                            const uint4 (&xr)[8][2], f32x4 &acc0, f32x4 &acc1)
{
    const TileStreams ts = tile_streams(B, 2, np, nU, nD);
    uint32_t ru = 0, rd = 0;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        if (p < npq) {
            uint32_t w[8];
            decode_panel_lds<B>(tile, ts, p, ru, rd, w);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8, xr[p][0]),
                __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3])), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8, xr[p][1]),
                __builtin_bit_cast(bf16x8, make_uint4(w[4], w[5], w[6], w[7])), acc1, 0, 0, 0);
        }
    }
}

// ---- B = 16: a half tile (4 panels) at a time.  Its 8 masks are read from the LDS copy of the tile
// (uniform address) together with the previous half's payload reads, then made scalar; all payload
// reads of a half are issued before its first decode ------------------------------------------------
struct HalfMasks {
    uint64_t u[4], d[4];
};

// LDS reads of DMA-filled memory are written as inline assembly on purpose: for an ordinary LDS
// load that may alias a pending global_load_lds the compiler inserts a wait for ALL pending DMA,
// which would cancel the prefetch distance.  Here the slot discipline (a slot is read only after the
// explicit vmcnt wait for its own DMA, and refilled only after its last read has returned) is the
// proof of ordering, and the reads are followed by one explicit lgkmcnt(0).
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
__device__ inline void lds_read_2xb128(u32x4_t &lo, u32x4_t &hi, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:16" : "=&v"(lo), "=&v"(hi) : "v"(addr));
}

// Four 16-byte {U, D} mask pairs, as read from LDS (identical in every lane).
struct RawMasks {
    u32x4_t v[4];
};

__device__ inline void lds_read_masks(RawMasks &mv, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:16\n\t"
                 "ds_read_b128 %2, %4 offset:32\n\tds_read_b128 %3, %4 offset:48"
                 : "=&v"(mv.v[0]), "=&v"(mv.v[1]), "=&v"(mv.v[2]), "=&v"(mv.v[3])
                 : "v"(addr));
}

// The four raw mask pairs into scalar registers.
__device__ inline void scalar_masks(const RawMasks &mv, HalfMasks &m)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // (the builtin returns a signed int: go through uint32_t before widening)
        const uint32_t ulo = __builtin_amdgcn_readfirstlane(mv.v[i].x), uhi = __builtin_amdgcn_readfirstlane(mv.v[i].y);
        const uint32_t dlo = __builtin_amdgcn_readfirstlane(mv.v[i].z), dhi = __builtin_amdgcn_readfirstlane(mv.v[i].w);
        const uint64_t u = (uint64_t(uhi) << 32) | ulo;
        const uint64_t d = (uint64_t(dhi) << 32) | dlo;
        m.u[i] = u;
        m.d[i] = d;
    }
}

// Decode + MFMA of panels P0 .. P0 + 3; also fetches the raw masks at next_masks (LDS address) for the
// half that follows, so that they arrive under the same wait as this half's payload.
template <int P0>
__device__ inline void process_half16(uint32_t tile_lds, const HalfMasks &m, uint32_t dense_off,
                                      uint32_t rec_off, uint32_t &ru, uint32_t &rd, const uint4 (&xr)[8][2],
                                      f32x4 &acc0, f32x4 &acc1, uint32_t next_masks, RawMasks &mv)
{
    uint32_t rec[4];
    u32x4_t wlo[4], whi[4];
    lds_read_masks(mv, next_masks);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        // Every lane reads (a lane without a UNIFIED block reads its neighbour's record and drops it
        // below): an unconditional read leaves no register copy between the read and the wait.
        rec[p] = lds_read_b32(tile_lds + rec_off + 4u * (ru + mbcnt64(m.u[p])));
        if (__builtin_amdgcn_inverse_ballot_w64(m.d[p]))
            lds_read_2xb128(wlo[p], whi[p], tile_lds + dense_off + 32u * (rd + mbcnt64(m.d[p])));
        ru += __popcll(m.u[p]);
        rd += __popcll(m.d[p]);
    }
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(rec[0]), "+v"(rec[1]), "+v"(rec[2]), "+v"(rec[3]), "+v"(wlo[0]), "+v"(wlo[1]),
                   "+v"(wlo[2]), "+v"(wlo[3]), "+v"(whi[0]), "+v"(whi[1]), "+v"(whi[2]), "+v"(whi[3]),
                   "+v"(mv.v[0]), "+v"(mv.v[1]), "+v"(mv.v[2]), "+v"(mv.v[3]));
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        if (!__builtin_amdgcn_inverse_ballot_w64(m.d[p])) {
            // record = magnitude (low half, sign bit clear) | permuted sign field (high half)
            const uint32_t rc = __builtin_amdgcn_inverse_ballot_w64(m.u[p]) ? rec[p] : 0u;
            const uint32_t qq = __builtin_amdgcn_perm(rc, rc, 0x01000100u);
            const uint32_t sw = __builtin_amdgcn_perm(rc, rc, 0x030c020cu);
            wlo[p].x = qq | (sw & 0x80008000u);
            wlo[p].y = qq | ((sw << 1) & 0x80008000u);
            wlo[p].z = qq | ((sw << 2) & 0x80008000u);
            wlo[p].w = qq | ((sw << 3) & 0x80008000u);
            whi[p].x = qq | ((sw << 4) & 0x80008000u);
            whi[p].y = qq | ((sw << 5) & 0x80008000u);
            whi[p].z = qq | ((sw << 6) & 0x80008000u);
            whi[p].w = qq | ((sw << 7) & 0x80008000u);
        }
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xr[P0 + p][0]),
                                                       __builtin_bit_cast(bf16x8, wlo[p]), acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xr[P0 + p][1]),
                                                       __builtin_bit_cast(bf16x8, whi[p]), acc1, 0, 0, 0);
    }
}

// The few layout numbers the kernel needs (32-bit, to keep scalar registers for the masks).
struct StreamGeom {
    uint32_t dir_off, streams_off;
    int32_t KT, NS, N, K;
};

template <int B, int NCH, int D, int SPI>
__global__ __launch_bounds__(512) void k_stream_bf16(StreamArgs a, StreamGeom L)
{
    constexpr int SLOT = NCH * 1024;
    constexpr int NSLOT = D + 1;
    __shared__ __attribute__((aligned(16))) uint8_t ring[8][NSLOT * SLOT];
    __shared__ __attribute__((aligned(16))) float red[2][8][SPI][64][4];

    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63, r = lane & 15, g4 = lane >> 4;
    const int chunk = blockIdx.y;
    const int kt = chunk * 8 + wave;
    const bool active = kt < L.KT;
    int np = 0;
    if (active) {
        const int left = (L.K + kPanelK - 1) / kPanelK - kt * kTilePanels;
        np = left < kTilePanels ? left : kTilePanels;
    }

    const int bb_lo = blockIdx.x * a.per_wg;
    int bb_hi = bb_lo + a.per_wg;
    if (bb_hi > a.nbatches) bb_hi = a.nbatches;
    if (bb_lo >= bb_hi) return;
    const int nb = bb_hi - bb_lo;
    const int nseq = nb * SPI;
    uint8_t *myring = ring[wave];

    // ---- directory window: lane l holds stream address, size and counts of sequence element qbase + l
    int qbase = 0;
    uint64_t q_addr = 0;
    uint32_t q_bytes = 0, q_cnt = 0, q_np = 0;
    auto refill = [&](int base) {
        qbase = base;
        const int qq = base + lane;
        const int bb = bb_lo + qq / SPI;
        const int gi = bb / a.nbpm;
        const int64_t strip = int64_t(bb % a.nbpm) * SPI + qq % SPI;
        const bool ok = active && qq < nseq && strip < L.NS;
        uint64_t blob = reinterpret_cast<uint64_t>(a.blob);
        if (a.blobs) blob = ((const __attribute__((address_space(1))) uint64_t *)a.blobs)[ok ? gi : 0];
        q_addr = blob;  // a valid 16 bytes for elements with nothing to fetch
        q_bytes = 16;
        q_cnt = 0;
        q_np = 0;
        if (ok) {
            g_cu32 *de = (g_cu32 *)(blob + L.dir_off + uint64_t(strip * L.KT + kt) * sizeof(DirEntry));
            const uint32_t off16 = de[0], cnt = de[1], next = de[2];
            q_addr = blob + L.streams_off + uint64_t(off16) * 16;
            q_bytes = (next - off16) * 16;
            q_cnt = cnt;  // nU | nD << 16
            q_np = uint32_t(np);
        }
        // Drain on every path: a load left pending here would turn each later read of the window
        // registers into a wait for all DMA prefetches as well.
        wait_vmcnt<0>();
    };
    auto entry_addr = [&](int e) {
        const uint32_t lo = __builtin_amdgcn_readlane(uint32_t(q_addr), e - qbase);
        const uint32_t hi = __builtin_amdgcn_readlane(uint32_t(q_addr >> 32), e - qbase);
        return (uint64_t(hi) << 32) | lo;
    };
    // ---- issue the NCH DMA instructions of sequence element qi into its ring slot
    auto issue = [&](int qi) {
        const uint64_t base = entry_addr(qi);
        const uint32_t bytes = __builtin_amdgcn_readlane(q_bytes, qi - qbase);
        const int slot = qi % NSLOT;
        const uint32_t last = bytes - 16;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            uint32_t off = uint32_t(c) * 1024u + uint32_t(lane) * 16u;
            off = off < last ? off : last;
            __builtin_amdgcn_global_load_lds((global_void_t *)(base + off),
                                             (lds_void_t *)(myring + slot * SLOT + c * 1024), 16, 0, 0);
        }
    };

    uint4 xr[8][2];
#pragma unroll
    for (int p = 0; p < 8; ++p) xr[p][0] = xr[p][1] = make_uint4(0, 0, 0, 0);
    int cur_g = -1;
    RawMasks mv{};  // raw masks of the half that is decoded next

    if (active) {
        refill(0);
        for (int qi = 0; qi < D && qi < nseq; ++qi) issue(qi);
        if constexpr (B == 16) {
            wait_vmcnt<0>();  // once per workgroup: tile 0 must have landed before its masks are read
            lds_read_masks(mv, lds_offset(myring));
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(mv.v[0]), "+v"(mv.v[1]), "+v"(mv.v[2]), "+v"(mv.v[3]));
        }
    }

    for (int bi = 0; bi < nb; ++bi) {
        const int bb = bb_lo + bi;
        const int gi = bb / a.nbpm;
        const int64_t strip0 = int64_t(bb % a.nbpm) * SPI;
        if (gi != cur_g && active) {
            cur_g = gi;
            const uint64_t X = a.Xs ? table_entry(a.Xs, gi) : reinterpret_cast<uint64_t>(a.X);
#pragma unroll
            for (int p = 0; p < 8; ++p)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int64_t k = int64_t(kt) * kTileK + p * kPanelK + 16 * g4 + 8 * h;
                    uint4 v = make_uint4(0, 0, 0, 0);
                    if (r < a.M && k + 8 <= L.K) {
                        const u32x4_t t = *(g_cu32x4 *)(X + uint64_t(int64_t(r) * a.ldx + k) * 2u);
                        v = make_uint4(t.x, t.y, t.z, t.w);
                    }
                    xr[p][h] = v;
                }
            // Drain here, once per matrix, so that no later use of xr needs a wait that would also
            // wait for the DMA prefetches in flight.
            wait_vmcnt<0>();
        }
#pragma unroll
        for (int s = 0; s < SPI; ++s) {
            f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
            if (active) {
                const int q = bi * SPI + s;
                const int qi = q + D;
                if (qi < nseq && qi >= qbase + 64) refill(q);  // keeps q .. q + 63, covers q, q + 1, q + D
                const uint32_t cnt = __builtin_amdgcn_readlane(q_cnt, q - qbase);
                const int npq = int(__builtin_amdgcn_readlane(q_np, q - qbase));
                // After this wait tiles q and q + 1 have landed (q + 1 because its first masks are
                // fetched while q is still being decoded).
                if (qi < nseq) {
                    issue(qi);
                    wait_vmcnt<(D - 1) * NCH>();
                } else {
                    wait_vmcnt<0>();
                }
                const uint8_t *tile = myring + (q % NSLOT) * SLOT;
                if constexpr (B == 16) {
                    const uint32_t dense_off = 128u, rec_off = dense_off + (cnt >> 16) * 32u;
                    uint32_t ru = 0, rd = 0;
                    const uint32_t tl = lds_offset(tile);
                    const uint32_t tl_next = lds_offset(myring + ((q + 1) % NSLOT) * SLOT);
                    HalfMasks sm;
                    scalar_masks(mv, sm);
                    process_half16<0>(tl, sm, dense_off, rec_off, ru, rd, xr, acc0, acc1, tl + 64u, mv);
                    scalar_masks(mv, sm);
                    process_half16<4>(tl, sm, dense_off, rec_off, ru, rd, xr, acc0, acc1, tl_next, mv);
                } else
                    process_tile_generic<B>(tile, np, npq, cnt & 0xffffu, cnt >> 16, xr, acc0, acc1);
            }
            *reinterpret_cast<f32x4 *>(red[bi & 1][wave][s][lane]) = acc0 + acc1;
        }
        lds_barrier();
        if (wave == (bi & 7)) {
            const uint64_t Y = a.Ys ? table_entry(a.Ys, gi) : reinterpret_cast<uint64_t>(a.Y);
#pragma unroll
            for (int s = 0; s < SPI; ++s) {
                // (asm reads for the same reason as the tile reads: no wait on the DMA in flight)
                f32x4 part[8];
#pragma unroll
                for (int w2 = 0; w2 < 8; ++w2)
                    asm volatile("ds_read_b128 %0, %1" : "=v"(part[w2]) : "v"(lds_offset(red[bi & 1][w2][s][lane])));
                asm volatile("s_waitcnt lgkmcnt(0)"
                             : "+v"(part[0]), "+v"(part[1]), "+v"(part[2]), "+v"(part[3]), "+v"(part[4]),
                               "+v"(part[5]), "+v"(part[6]), "+v"(part[7]));
                f32x4 t = part[0];  // waves without a tile column wrote zeros
#pragma unroll
                for (int w2 = 1; w2 < 8; ++w2) t += part[w2];
                const int64_t n = (strip0 + s) * kStripRows + r;
                if (n < L.N) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int m = 4 * g4 + v;
                        if (m >= a.M) continue;
                        if (a.Ypart)
                            ((g_float *)a.Ypart)[((int64_t(chunk) * a.G + gi) * a.M + m) * L.N + n] = t[v];
                        else if (a.ydtype == MUW_F32)
                            ((g_float *)Y)[int64_t(m) * a.ldy + n] = t[v];
                        else
                            ((g_u16 *)Y)[int64_t(m) * a.ldy + n] = f32_to_bf16_rne(t[v]);
                    }
                }
            }
        }
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

template <int B, int NCH, int D>
muw_status launch_stream_variant(StreamArgs a, const Layout &L, int64_t nstrips_total, hipStream_t st)
{
    const StreamGeom geom{uint32_t(L.dir_off), uint32_t(L.streams_off), int32_t(L.KT), int32_t(L.NS),
                          int32_t(L.N), int32_t(L.K)};
    const int cus = device_cus();
    // two strips per barrier when there is enough work to keep every compute unit busy anyway
    const bool spi2 = (L.NS + 1) / 2 * int64_t(a.G) >= 2 * int64_t(cus);
    const int SPI = spi2 ? 2 : 1;
    a.nbpm = int((L.NS + SPI - 1) / SPI);
    a.nbatches = a.nbpm * a.G;
    int grid = a.nbatches < cus ? a.nbatches : cus;
    a.per_wg = (a.nbatches + grid - 1) / grid;
    grid = (a.nbatches + a.per_wg - 1) / a.per_wg;
    dim3 g(unsigned(grid), unsigned(a.nchunk), 1);
    (void)nstrips_total;
    if (spi2)
        k_stream_bf16<B, NCH, D, 2><<<g, 512, 0, st>>>(a, geom);
    else
        k_stream_bf16<B, NCH, D, 1><<<g, 512, 0, st>>>(a, geom);
    return hip_status(hipGetLastError());
}

template <int B>
muw_status launch_stream_b(StreamArgs a, const Layout &L, int nch, hipStream_t st)
{
    const int64_t total = L.NS * int64_t(a.G);
    switch (nch) {
    case 1:
    case 2: return launch_stream_variant<B, 2, 6>(a, L, total, st);
    case 3: return launch_stream_variant<B, 3, 4>(a, L, total, st);
    case 4: return launch_stream_variant<B, 4, 3>(a, L, total, st);
    default: return MUW_EUNSUPPORTED;
    }
}

}  // namespace

// Can the streaming kernel take this problem?  (bf16, M <= 16, 16-byte aligned activation rows, tile
// streams that fit the LDS ring.)
bool stream_gemm_applicable(const muw_desc &d, const Layout &L, const GemmArgs &a)
{
    if (d.wdtype != MUW_BF16 || a.M > 16 || a.M < 1) return false;
    if (d.max_tile_bytes <= 0 || d.max_tile_bytes > 4096) return false;
    if (L.K % 8 != 0 || a.ldx % 8 != 0) return false;
    if (!a.blobs && (reinterpret_cast<uintptr_t>(a.X) & 15u)) return false;
    if (a.G > 32767 || L.NS * int64_t(a.G) > (int64_t(1) << 30)) return false;
    return true;
}

size_t stream_gemm_workspace_bytes(const Layout &L, int64_t M, int G)
{
    const int64_t nchunk = (L.KT + 7) / 8;
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
    a.ldx = g.ldx;
    a.ldy = g.ldy;
    a.ydtype = g.ydtype;
    a.nchunk = int32_t((L.KT + 7) / 8);
    a.Ypart = a.nchunk > 1 ? static_cast<float *>(ws) : nullptr;
    const int nch = (d.max_tile_bytes + 1023) / 1024;
    muw_status rc;
    switch (d.B) {
    case 4: rc = launch_stream_b<4>(a, L, nch, st); break;
    case 8: rc = launch_stream_b<8>(a, L, nch, st); break;
    case 16: rc = launch_stream_b<16>(a, L, nch, st); break;
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
