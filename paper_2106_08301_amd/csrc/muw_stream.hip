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

// The executing lane's 16 weights of panel p of the tile stream that sits in LDS at `tile`.
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
        if (__builtin_amdgcn_inverse_ballot_w64(mu)) {
            q = reinterpret_cast<const uint16_t *>(tile + ts.mag_off)[rku];
            s = load_sign_field<B>(tile + ts.sign_off, rku);
        }
        decode_block_bf16<B>(q, s, w + j * (B / 2));
        if (__builtin_amdgcn_inverse_ballot_w64(md)) {
            const uint32_t *src = reinterpret_cast<const uint32_t *>(tile + ts.dense_off) + rkd * (B / 2);
#pragma unroll
            for (int d = 0; d < B / 2; ++d) w[j * (B / 2) + d] = src[d];
        }
    }
}

template <int B, int NCH, int D, int SPI>
__global__ __launch_bounds__(512) void k_stream_bf16(StreamArgs a, Layout L)
{
    constexpr int SLOT = NCH * 1024;
    constexpr int NSLOT = D + 1;
    __shared__ __attribute__((aligned(16))) uint8_t ring[8][NSLOT * SLOT];
    __shared__ __attribute__((aligned(16))) float red[2][8][SPI][64][4];
    __shared__ uint32_t slot_meta[8][NSLOT][2];

    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63, r = lane & 15, g4 = lane >> 4;
    const int chunk = blockIdx.y;
    const int kt = chunk * 8 + wave;
    const bool active = kt < L.KT;
    const int np = active ? panels_in_tile(L, kt) : 0;
    const int nact = (L.KT - chunk * 8) < 8 ? int(L.KT - chunk * 8) : 8;

    const int bb_lo = blockIdx.x * a.per_wg;
    int bb_hi = bb_lo + a.per_wg;
    if (bb_hi > a.nbatches) bb_hi = a.nbatches;
    if (bb_lo >= bb_hi) return;
    const int nb = bb_hi - bb_lo;
    const int nseq = nb * SPI;
    uint8_t *myring = ring[wave];

    // ---- directory queue: lane l holds the stream address and counts of sequence element qbase + l
    uint64_t q_addr = 0;
    uint32_t q_bytes = 0, q_cnt = 0, q_np = 0;
    auto refill = [&](int qbase) {
        const int qq = qbase + lane;
        const int bb = bb_lo + qq / SPI;
        const int gi = bb / a.nbpm;
        const int64_t strip = int64_t(bb % a.nbpm) * SPI + qq % SPI;
        const bool ok = active && qq < nseq && strip < L.NS;
        const uint8_t *blob = a.blob;
        if (a.blobs) blob = static_cast<const uint8_t *>(a.blobs[ok ? gi : 0]);
        q_addr = reinterpret_cast<uint64_t>(blob);  // a valid 16 bytes for lanes with nothing to fetch
        q_bytes = 16;
        q_cnt = 0;
        q_np = 0;
        if (ok) {
            const DirEntry *de = reinterpret_cast<const DirEntry *>(blob + L.dir_off) + strip * L.KT + kt;
            const DirEntry e0 = de[0];
            const uint32_t next = de[1].off16;
            q_addr = reinterpret_cast<uint64_t>(blob + L.streams_off) + uint64_t(e0.off16) * 16;
            q_bytes = (next - e0.off16) * 16;
            q_cnt = uint32_t(e0.nU) | (uint32_t(e0.nD) << 16);
            q_np = uint32_t(np);
        }
    };
    // ---- issue the NCH DMA instructions of sequence element qi into its ring slot
    auto issue = [&](int qi) {
        const int src_lane = qi & 63;
        const uint32_t alo = __builtin_amdgcn_readlane(uint32_t(q_addr), src_lane);
        const uint32_t ahi = __builtin_amdgcn_readlane(uint32_t(q_addr >> 32), src_lane);
        const uint32_t bytes = __builtin_amdgcn_readlane(q_bytes, src_lane);
        const uint32_t cnt = __builtin_amdgcn_readlane(q_cnt, src_lane);
        const uint32_t npq = __builtin_amdgcn_readlane(q_np, src_lane);
        const uint64_t base = (uint64_t(ahi) << 32) | alo;
        const int slot = qi % NSLOT;
        if (lane == 0) {
            slot_meta[wave][slot][0] = cnt;
            slot_meta[wave][slot][1] = npq;
        }
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

    if (active) {
        refill(0);
        for (int qi = 0; qi < D && qi < nseq; ++qi) issue(qi);
    }

    for (int bi = 0; bi < nb; ++bi) {
        const int bb = bb_lo + bi;
        const int gi = bb / a.nbpm;
        const int64_t strip0 = int64_t(bb % a.nbpm) * SPI;
        if (gi != cur_g && active) {
            cur_g = gi;
            const uint16_t *X = a.Xs ? static_cast<const uint16_t *>(a.Xs[gi]) : a.X;
#pragma unroll
            for (int p = 0; p < 8; ++p)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int64_t k = int64_t(kt) * kTileK + p * kPanelK + 16 * g4 + 8 * h;
                    uint4 v = make_uint4(0, 0, 0, 0);
                    if (r < a.M && k + 8 <= L.K) v = *reinterpret_cast<const uint4 *>(X + int64_t(r) * a.ldx + k);
                    xr[p][h] = v;
                }
            // Drain here, once per matrix, so that no later use of xr needs a wait that would also
            // wait for the DMA prefetches in flight.
            wait_vmcnt<0>();
        }
        f32x4 acc[SPI];
#pragma unroll
        for (int s = 0; s < SPI; ++s) {
            acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (active) {
                const int q = bi * SPI + s;
                const int qi = q + D;
                if (qi < nseq) {
                    if ((qi & 63) == 0) refill(qi);
                    issue(qi);
                    wait_vmcnt<D * NCH>();
                } else {
                    wait_vmcnt<0>();
                }
                const int slot = q % NSLOT;
                const uint8_t *tile = myring + slot * SLOT;
                const uint32_t cnt = __builtin_amdgcn_readfirstlane(slot_meta[wave][slot][0]);
                const int npq = __builtin_amdgcn_readfirstlane(slot_meta[wave][slot][1]);
                const TileStreams ts = tile_streams(B, 2, np, cnt & 0xffffu, cnt >> 16);
                uint32_t ru = 0, rd = 0;
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    if (p < npq) {
                        uint32_t w[8];
                        decode_panel_lds<B>(tile, ts, p, ru, rd, w);
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const uint4 b = make_uint4(w[4 * h], w[4 * h + 1], w[4 * h + 2], w[4 * h + 3]);
                            acc[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(bf16x8, xr[p][h]), __builtin_bit_cast(bf16x8, b), acc[s], 0, 0, 0);
                        }
                    }
                }
            }
            *reinterpret_cast<f32x4 *>(red[bi & 1][wave][s][lane]) = acc[s];
        }
        __syncthreads();
        if (wave == (bi & 7)) {
#pragma unroll
            for (int s = 0; s < SPI; ++s) {
                f32x4 t = *reinterpret_cast<const f32x4 *>(red[bi & 1][0][s][lane]);
                for (int w2 = 1; w2 < nact; ++w2) t += *reinterpret_cast<const f32x4 *>(red[bi & 1][w2][s][lane]);
                const int64_t n = (strip0 + s) * kStripRows + r;
                if (n < L.N) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int m = 4 * g4 + v;
                        if (m >= a.M) continue;
                        if (a.Ypart) {
                            a.Ypart[((int64_t(chunk) * a.G + gi) * a.M + m) * L.N + n] = t[v];
                        } else {
                            void *Y = a.Ys ? a.Ys[gi] : a.Y;
                            if (a.ydtype == MUW_F32)
                                static_cast<float *>(Y)[int64_t(m) * a.ldy + n] = t[v];
                            else
                                static_cast<uint16_t *>(Y)[int64_t(m) * a.ldy + n] = f32_to_bf16_rne(t[v]);
                        }
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
        k_stream_bf16<B, NCH, D, 2><<<g, 512, 0, st>>>(a, L);
    else
        k_stream_bf16<B, NCH, D, 1><<<g, 512, 0, st>>>(a, L);
    return hip_status(hipGetLastError());
}

template <int B>
muw_status launch_stream_b(StreamArgs a, const Layout &L, int nch, hipStream_t st)
{
    const int64_t total = L.NS * int64_t(a.G);
    switch (nch) {
    case 1:
    case 2: return launch_stream_variant<B, 2, 5>(a, L, total, st);
    case 3: return launch_stream_variant<B, 3, 3>(a, L, total, st);
    case 4: return launch_stream_variant<B, 4, 2>(a, L, total, st);
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
