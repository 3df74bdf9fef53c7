// muw_unify.hip -- Unify() (Sec. 3.1, Sec. 3.3 Eq. 6) for a free two-dimensional block shape [BK, BN], written
// out dense: the Q-step of the training loop (Alg. 1, step 6) and the compression of Sec. 4.3 for any of the
// 2-D shapes of Table 1, without a packed format behind it.
//
// Compile with -ffp-contract=off: the block scores decide the selection by their exact fp64 bit patterns.
// Inside a block the sums run over its rows in order and, inside a row, over k in order.
#include "muw_decode.hpp"
#include "muw_internal.hpp"

namespace muw {

namespace {

struct WsU {
    uint64_t key_p, key_u, q, tags, flag, sel, total;
};

WsU carve(int64_t NB)
{
    WsU w;
    uint64_t off = 0;
    w.key_p = off;
    off = align16(off + uint64_t(NB) * 8);
    w.key_u = off;
    off = align16(off + uint64_t(NB) * 8);
    w.q = off;
    off = align16(off + uint64_t(NB) * 8);
    w.tags = off;
    off = align16(off + uint64_t(NB));
    w.flag = off;
    off = align16(off + 16);
    w.sel = off;
    off = align16(off + select_workspace_bytes(NB));
    w.total = off;
    return w;
}

__device__ inline double widen(float v) { return double(v); }
__device__ inline double widen(bf16_t v) { return double(__uint_as_float(uint32_t(v.bits) << 16)); }
__device__ inline float to_storage(float, double q) { return float(q); }
__device__ inline bf16_t to_storage(bf16_t, double q) { return bf16_t{f64_to_bf16_rne(q)}; }
__device__ inline float negated(float v) { return -v; }
__device__ inline bf16_t negated(bf16_t v) { return bf16_t{uint16_t(v.bits ^ 0x8000u)}; }

// One thread per block: q = mean |w|, e_p = sum w^2, e_u = sum (|w| - q)^2 in fp64.
template <typename T>
__global__ __launch_bounds__(256) void k_unify_scores(const T *W, int64_t K, int64_t KB, int64_t NB, int BK, int BN,
                                                      uint64_t *key_p, uint64_t *key_u, double *q_out, uint32_t *flag)
{
    const int64_t j = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (j >= NB) return;
    const T *base = W + (j / KB) * BN * K + (j % KB) * BK;
    bool bad = false;
    double s1 = 0.0;
    for (int r = 0; r < BN; ++r)
        for (int l = 0; l < BK; ++l) {
            const double w = widen(base[r * K + l]);
            bad |= !isfinite(w);
            s1 = s1 + fabs(w);
        }
    const double q = s1 / double(BK * BN);
    double e_p = 0.0, e_u = 0.0;
    for (int r = 0; r < BN; ++r)
        for (int l = 0; l < BK; ++l) {
            const double w = widen(base[r * K + l]);
            const double sq = w * w;
            e_p = e_p + sq;
        }
    for (int r = 0; r < BN; ++r)
        for (int l = 0; l < BK; ++l) {
            const double d = fabs(widen(base[r * K + l])) - q;
            const double dd = d * d;
            e_u = e_u + dd;
        }
    key_p[j] = uint64_t(__double_as_longlong(e_p));
    key_u[j] = uint64_t(__double_as_longlong(e_u));
    q_out[j] = q;
    if (bad) atomicOr(flag, 1u);
}

// One thread per weight: +-q^ in UNIFIED blocks (Eq. 2: w >= 0, -0.0 included, maps to +q^), 0 in PRUNED ones,
// the weight itself elsewhere; the block's first weight also writes the tag and the magnitude.
template <typename T>
__global__ __launch_bounds__(256) void k_unify_project(const T *W, int64_t N, int64_t K, int64_t KB, int BK, int BN,
                                                       const uint8_t *tags, const double *q, uint8_t *tags_out,
                                                       T *mags_out, T *What)
{
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= N * K) return;
    const int64_t n = i / K, k = i % K;
    const int64_t j = (n / BN) * KB + k / BK;
    const uint8_t tag = tags[j];
    const T w = W[i];
    T out = w, mag = T{};
    if (tag == MUW_TAG_PRUNED) {
        out = T{};
    } else if (tag == MUW_TAG_UNIFIED) {
        mag = to_storage(T{}, q[j]);
        out = widen(w) < 0.0 ? negated(mag) : mag;
    }
    if (What) What[i] = out;
    if (n % BN == 0 && k % BK == 0) {
        if (tags_out) tags_out[j] = tag;
        if (mags_out) mags_out[j] = mag;
    }
}

template <typename T>
muw_status unify_typed(int64_t N, int64_t K, int BK, int BN, const void *W, int64_t n_u, int64_t n_p, uint8_t *tags_out,
                       void *mags_out, void *What, uint8_t *ws, hipStream_t st, bool *nonfinite)
{
    const int64_t KB = K / BK, NB = (N / BN) * KB;
    const WsU w = carve(NB);
    uint64_t *key_p = reinterpret_cast<uint64_t *>(ws + w.key_p), *key_u = reinterpret_cast<uint64_t *>(ws + w.key_u);
    double *q = reinterpret_cast<double *>(ws + w.q);
    uint8_t *tags = ws + w.tags;
    uint32_t *flag = reinterpret_cast<uint32_t *>(ws + w.flag);
    if (hipMemsetAsync(tags, MUW_TAG_DENSE, size_t(NB), st) != hipSuccess) return MUW_EHIP;
    if (hipMemsetAsync(flag, 0, 16, st) != hipSuccess) return MUW_EHIP;
    k_unify_scores<T><<<unsigned((NB + 255) / 256), 256, 0, st>>>(static_cast<const T *>(W), K, KB, NB, BK, BN, key_p,
                                                                  key_u, q, flag);
    muw_status rc = select_k_smallest(key_p, NB, n_p, ws + w.sel, tags, MUW_TAG_PRUNED, key_u, 1, st);
    if (rc != MUW_OK) return rc;
    rc = select_k_smallest(key_u, NB, n_u, ws + w.sel, tags, MUW_TAG_UNIFIED, nullptr, 0, st);
    if (rc != MUW_OK) return rc;
    k_unify_project<T><<<unsigned((N * K + 255) / 256), 256, 0, st>>>(static_cast<const T *>(W), N, K, KB, BK, BN, tags,
                                                                      q, tags_out, static_cast<T *>(mags_out),
                                                                      static_cast<T *>(What));
    if (hipGetLastError() != hipSuccess) return MUW_EHIP;
    uint32_t bad = 0;
    if (hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, st) != hipSuccess) return MUW_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return MUW_EHIP;
    *nonfinite = bad != 0;
    return MUW_OK;
}

}  // namespace

size_t unify_workspace_bytes(int64_t NB) { return size_t(carve(NB).total); }

muw_status launch_unify(int64_t N, int64_t K, int BK, int BN, const void *W, int dtype, int64_t n_u, int64_t n_p,
                        uint8_t *tags_out, void *mags_out, void *What, void *ws, hipStream_t st, bool *nonfinite)
{
    if (dtype == MUW_BF16)
        return unify_typed<bf16_t>(N, K, BK, BN, W, n_u, n_p, tags_out, mags_out, What, static_cast<uint8_t *>(ws), st,
                                   nonfinite);
    return unify_typed<float>(N, K, BK, BN, W, n_u, n_p, tags_out, mags_out, What, static_cast<uint8_t *>(ws), st,
                              nonfinite);
}

}  // namespace muw
