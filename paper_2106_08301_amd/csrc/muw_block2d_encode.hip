// muw_block2d_encode.hip -- Unify() (Sec. 3.1, Sec. 3.3 Eq. 6) for [16, 32] blocks and the packing of its
// result into the layout of muw_block2d.hpp; export and decode of that layout.
//
// Compile with -ffp-contract=off: the block scores decide the selection by their exact fp64 bit patterns.
// Inside a block the sums run over the 32 rows in order and, inside a row, over its 16 weights in order.
#include "muw_block2d.hpp"
#include "muw_decode.hpp"

namespace muw {

namespace {

struct Ws2 {
    uint64_t key_p, key_u, q, tags, rank, cnt_u, cnt_d, flag, sel, total;
};

Ws2 carve(const Layout2 &L)
{
    Ws2 w;
    const uint64_t NB = uint64_t(L.NB);
    uint64_t off = 0;
    w.key_p = off;
    off = align16(off + NB * 8);
    w.key_u = off;
    off = align16(off + NB * 8);
    w.q = off;
    off = align16(off + NB * 8);
    w.tags = off;
    off = align16(off + NB);
    w.rank = off;
    off = align16(off + NB * 4);
    w.cnt_u = off;
    off = align16(off + uint64_t(L.NS + 1) * 4);
    w.cnt_d = off;
    off = align16(off + uint64_t(L.NS + 1) * 4);
    w.flag = off;
    off = align16(off + 16);
    w.sel = off;
    off = align16(off + select_workspace_bytes(L.NB));
    w.total = off;
    return w;
}

__device__ inline double widen_bf16(uint16_t bits) { return double(__uint_as_float(uint32_t(bits) << 16)); }

// One thread per block: q = mean |w|, e_p = sum w^2, e_u = sum (|w| - q)^2 in fp64, rows outer, k inner.
__global__ __launch_bounds__(256) void k_scores2d(const uint16_t *W, int64_t K, int64_t KC, int64_t NB,
                                                  uint64_t *key_p, uint64_t *key_u, double *q_out, uint32_t *flag)
{
    const int64_t j = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (j >= NB) return;
    const uint16_t *base = W + (j / KC) * kB2N * K + (j % KC) * kB2K;
    bool bad = false;
    double s1 = 0.0;
    for (int r = 0; r < kB2N; ++r)
        for (int l = 0; l < kB2K; ++l) {
            const double w = widen_bf16(base[r * K + l]);
            bad |= !isfinite(w);
            s1 = s1 + fabs(w);
        }
    const double q = s1 / double(kB2K * kB2N);
    double e_p = 0.0, e_u = 0.0;
    for (int r = 0; r < kB2N; ++r)
        for (int l = 0; l < kB2K; ++l) {
            const double w = widen_bf16(base[r * K + l]);
            const double sq = w * w;
            e_p = e_p + sq;
        }
    for (int r = 0; r < kB2N; ++r)
        for (int l = 0; l < kB2K; ++l) {
            const double d = fabs(widen_bf16(base[r * K + l])) - q;
            const double dd = d * d;
            e_u = e_u + dd;
        }
    key_p[j] = uint64_t(__double_as_longlong(e_p));
    key_u[j] = uint64_t(__double_as_longlong(e_u));
    q_out[j] = q;
    if (bad) atomicOr(flag, 1u);
}

// One thread per strip: the two bitmaps, each surviving block's rank inside its strip, the strip's counts.
__global__ __launch_bounds__(256) void k_strip_walk2d(const uint8_t *tags, Layout2 L, uint8_t *blob, uint32_t *rank,
                                                      uint32_t *cnt_u, uint32_t *cnt_d)
{
    const int64_t s = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (s >= L.NS) return;
    uint64_t *present = reinterpret_cast<uint64_t *>(blob + L.present_off) + s * L.W64;
    uint64_t *dense = reinterpret_cast<uint64_t *>(blob + L.densemap_off) + s * L.W64;
    uint32_t u = 0, d = 0;
    for (int64_t g = 0; g < L.W64; ++g) {
        uint64_t pm = 0, dm = 0;
        for (int b = 0; b < 64; ++b) {
            const int64_t kc = g * 64 + b;
            if (kc >= L.KC) break;
            const int64_t j = s * L.KC + kc;
            const uint8_t t = tags[j];
            if (t == MUW_TAG_UNIFIED) {
                rank[j] = u++;
                pm |= uint64_t(1) << b;
            } else if (t == MUW_TAG_DENSE) {
                rank[j] = d++;
                pm |= uint64_t(1) << b;
                dm |= uint64_t(1) << b;
            }
        }
        present[g] = pm;
        dense[g] = dm;
    }
    cnt_u[s] = u;
    cnt_d[s] = d;
}

// Header and directory (cnt_u / cnt_d hold exclusive prefix sums by now, entry NS = the totals).
__global__ __launch_bounds__(256) void k_header2d(Layout2 L, uint8_t *blob, const uint32_t *cnt_u, const uint32_t *cnt_d)
{
    const int64_t s = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (s == 0) {
        uint32_t *h32 = reinterpret_cast<uint32_t *>(blob);
        int64_t *h64 = reinterpret_cast<int64_t *>(blob);
        h32[0] = kMagic2;
        h32[1] = (uint32_t(kB2N) << 16) | uint32_t(kB2K);
        h64[1] = L.N;
        h64[2] = L.K;
        h64[3] = L.n_u;
        h64[4] = L.n_d;
        h64[5] = int64_t(L.total);
    }
    if (s <= L.NS) {
        uint32_t *dir = reinterpret_cast<uint32_t *>(blob + L.dir_off) + 2 * s;
        dir[0] = cnt_u[s];
        dir[1] = cnt_d[s];
    }
}

// One wavefront per block: lane l holds W[32 s + l % 32][16 kc + 8 (l / 32) .. + 7].
__global__ __launch_bounds__(256) void k_pack2d(const uint16_t *W, const uint8_t *tags, const uint32_t *rank,
                                                const double *q, const uint32_t *cnt_u, const uint32_t *cnt_d,
                                                Layout2 L, uint8_t *blob)
{
    const int64_t j = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (j >= L.NB) return;
    const uint8_t tag = tags[j];
    if (tag == MUW_TAG_PRUNED) return;  // nothing is stored for a pruned block (Sec. 3.1)
    const int lane = threadIdx.x & 63;
    const int64_t s = j / L.KC, kc = j % L.KC;
    const uint16_t *src = W + (s * kB2N + (lane & 31)) * L.K + kc * kB2K + (lane >> 5) * 8;
    const uint4 raw = *reinterpret_cast<const uint4 *>(src);
    if (tag == MUW_TAG_DENSE) {
        uint8_t *dst = blob + L.dense_off + (uint64_t(cnt_d[s]) + rank[j]) * 1024u + uint32_t(lane) * 16u;
        *reinterpret_cast<uint4 *>(dst) = raw;
        return;
    }
    const uint64_t g = uint64_t(cnt_u[s]) + rank[j];
    const uint32_t v[4] = {raw.x, raw.y, raw.z, raw.w};
    uint32_t byte = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t bits = (v[i >> 1] >> ((i & 1) * 16)) & 0xffffu;
        // Eq. 2: w >= 0 (which includes -0.0) maps to +q
        const bool neg = (bits & 0x8000u) && (bits & 0x7fffu);
        if (neg) byte |= 1u << ((i >> 1) + 4 * (i & 1));
    }
    (blob + L.signs_off + g * 64u)[lane] = uint8_t(byte);
    if (lane == 0) reinterpret_cast<uint16_t *>(blob + L.mags_off)[g] = f64_to_bf16_rne(q[j]);
}

// Tag and payload rank of block (s, kc) from the bitmaps.
struct BlockRef {
    int tag;
    uint64_t rank;
};
__device__ inline BlockRef find_block(const uint8_t *blob, const Layout2 &L, int64_t s, int64_t kc)
{
    const uint64_t *present = reinterpret_cast<const uint64_t *>(blob + L.present_off) + s * L.W64;
    const uint64_t *dense = reinterpret_cast<const uint64_t *>(blob + L.densemap_off) + s * L.W64;
    const uint32_t *dir = reinterpret_cast<const uint32_t *>(blob + L.dir_off) + 2 * s;
    const int64_t g = kc / 64;
    const int b = int(kc % 64);
    BlockRef r;
    if (!((present[g] >> b) & 1)) {
        r.tag = MUW_TAG_PRUNED;
        r.rank = 0;
        return r;
    }
    const bool is_dense = (dense[g] >> b) & 1;
    uint64_t before = 0;
    for (int64_t i = 0; i <= g; ++i) {
        uint64_t m = is_dense ? dense[i] : (present[i] & ~dense[i]);
        if (i == g) m &= (uint64_t(1) << b) - 1;
        before += uint64_t(__popcll(m));
    }
    r.tag = is_dense ? MUW_TAG_DENSE : MUW_TAG_UNIFIED;
    r.rank = uint64_t(dir[is_dense ? 1 : 0]) + before;
    return r;
}

__global__ __launch_bounds__(256) void k_export2d(const uint8_t *blob, Layout2 L, uint8_t *tags, uint16_t *mags)
{
    const int64_t j = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (j >= L.NB) return;
    const BlockRef r = find_block(blob, L, j / L.KC, j % L.KC);
    if (tags) tags[j] = uint8_t(r.tag);
    if (mags) mags[j] = r.tag == MUW_TAG_UNIFIED ? reinterpret_cast<const uint16_t *>(blob + L.mags_off)[r.rank] : 0;
}

__global__ __launch_bounds__(256) void k_decode2d(const uint8_t *blob, Layout2 L, uint16_t *What)
{
    const int64_t j = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (j >= L.NB) return;
    const int lane = threadIdx.x & 63;
    const int64_t s = j / L.KC, kc = j % L.KC;
    const BlockRef r = find_block(blob, L, s, kc);
    uint4 out = make_uint4(0, 0, 0, 0);
    if (r.tag == MUW_TAG_DENSE) {
        out = *reinterpret_cast<const uint4 *>(blob + L.dense_off + r.rank * 1024u + uint32_t(lane) * 16u);
    } else if (r.tag == MUW_TAG_UNIFIED) {
        const uint32_t q = reinterpret_cast<const uint16_t *>(blob + L.mags_off)[r.rank];
        const uint32_t byte = (blob + L.signs_off + r.rank * 64u)[lane];
        uint32_t v[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t lo = q | (((byte >> d) & 1u) << 15);
            const uint32_t hi = q | (((byte >> (d + 4)) & 1u) << 15);
            v[d] = lo | (hi << 16);
        }
        out = make_uint4(v[0], v[1], v[2], v[3]);
    }
    uint16_t *dst = What + (s * kB2N + (lane & 31)) * L.K + kc * kB2K + (lane >> 5) * 8;
    *reinterpret_cast<uint4 *>(dst) = out;
}

}  // namespace

size_t block2d_encode_workspace(const Layout2 &L) { return size_t(carve(L).total); }

muw_status launch_block2d_encode(const Layout2 &L, const void *W, int64_t n_u, int64_t n_p, void *blob_v, void *ws_v,
                                 hipStream_t st, bool *nonfinite)
{
    const Ws2 w = carve(L);
    uint8_t *ws = static_cast<uint8_t *>(ws_v), *blob = static_cast<uint8_t *>(blob_v);
    uint64_t *key_p = reinterpret_cast<uint64_t *>(ws + w.key_p), *key_u = reinterpret_cast<uint64_t *>(ws + w.key_u);
    double *q = reinterpret_cast<double *>(ws + w.q);
    uint8_t *tags = ws + w.tags;
    uint32_t *rank = reinterpret_cast<uint32_t *>(ws + w.rank);
    uint32_t *cnt_u = reinterpret_cast<uint32_t *>(ws + w.cnt_u), *cnt_d = reinterpret_cast<uint32_t *>(ws + w.cnt_d);
    uint32_t *flag = reinterpret_cast<uint32_t *>(ws + w.flag);

    if (hipMemsetAsync(blob, 0, size_t(L.total), st) != hipSuccess) return MUW_EHIP;
    if (hipMemsetAsync(tags, MUW_TAG_DENSE, size_t(L.NB), st) != hipSuccess) return MUW_EHIP;
    if (hipMemsetAsync(ws + w.cnt_u, 0, size_t(w.sel - w.cnt_u), st) != hipSuccess) return MUW_EHIP;

    const unsigned grid_blocks = unsigned((L.NB + 255) / 256);
    k_scores2d<<<grid_blocks, 256, 0, st>>>(static_cast<const uint16_t *>(W), L.K, L.KC, L.NB, key_p, key_u, q, flag);
    muw_status rc = select_k_smallest(key_p, L.NB, n_p, ws + w.sel, tags, MUW_TAG_PRUNED, key_u, 1, st);
    if (rc != MUW_OK) return rc;
    rc = select_k_smallest(key_u, L.NB, n_u, ws + w.sel, tags, MUW_TAG_UNIFIED, nullptr, 0, st);
    if (rc != MUW_OK) return rc;

    k_strip_walk2d<<<unsigned((L.NS + 255) / 256), 256, 0, st>>>(tags, L, blob, rank, cnt_u, cnt_d);
    launch_exclusive_scan(cnt_u, L.NS + 1, st);
    launch_exclusive_scan(cnt_d, L.NS + 1, st);
    k_header2d<<<unsigned((L.NS + 1 + 255) / 256), 256, 0, st>>>(L, blob, cnt_u, cnt_d);
    k_pack2d<<<unsigned((L.NB + 3) / 4), 256, 0, st>>>(static_cast<const uint16_t *>(W), tags, rank, q, cnt_u, cnt_d, L,
                                                        blob);
    if (hipGetLastError() != hipSuccess) return MUW_EHIP;
    uint32_t bad = 0;
    if (hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, st) != hipSuccess) return MUW_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return MUW_EHIP;
    *nonfinite = bad != 0;
    return MUW_OK;
}

muw_status launch_block2d_export(const Layout2 &L, const void *blob, uint8_t *tags, void *mags, hipStream_t st)
{
    k_export2d<<<unsigned((L.NB + 255) / 256), 256, 0, st>>>(static_cast<const uint8_t *>(blob), L, tags,
                                                             static_cast<uint16_t *>(mags));
    return hip_status(hipGetLastError());
}

muw_status launch_block2d_decode(const Layout2 &L, const void *blob, void *What, hipStream_t st)
{
    k_decode2d<<<unsigned((L.NB + 3) / 4), 256, 0, st>>>(static_cast<const uint8_t *>(blob), L,
                                                         static_cast<uint16_t *>(What));
    return hip_status(hipGetLastError());
}

}  // namespace muw
