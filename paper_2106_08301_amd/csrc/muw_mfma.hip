// muw_mfma.hip -- the compute-bound regime (many activation rows, bf16): Y = X * W^^T as an LDS-tiled
// MFMA GEMM whose B tile is produced by decoding the compressed panels (paper Sec. 3.2: the layer is a
// blocked GEMM; pruned blocks decode to nothing read from memory, unified blocks to +-q).
//
// Workgroup = 4 wavefronts, macro tile TM x 128 x 64 (TM = 128 or 256), one panel column (64 k) per
// step:
//   A tile  X[m0 .. m0+TM)[k0 .. k0+64) : 16-byte global loads -> LDS rows of 128 bytes whose 16-byte
//           chunks are XOR-swizzled with the row number (conflict-free 128-bit MFMA operand reads)
//   B tile  8 strips x 1 panel: each wave decodes 2 strip-panels straight from the blob (masks ->
//           payload index by v_mbcnt, one shift + bit-select per bf16 pair) and writes the lane's 16
//           weights as two swizzled 16-byte chunks of row n
//   MFMA    waves in a 2 x 2 grid, wave tile (TM/2) x 64: per step 2 x (TM/32) x 4 v_mfma_f32_16x16x32_bf16
// The k order inside a panel is the decode order (lane group g owns k = 16 g .. 16 g + 15; MFMA h takes
// 8 h .. 8 h + 7 of them), applied identically to both operands.  fp32 accumulation, no split-K: the
// result is bitwise reproducible.  Two workgroups per compute unit hide each other's load/decode phase.
#include "muw_decode.hpp"
#include "muw_internal.hpp"

namespace muw {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kTN = 128;  // output columns (rows of W) per workgroup

struct TileGemmArgs {
    const uint8_t *blob;
    const uint16_t *X;
    void *Y;
    int64_t M, ldx, ldy;
    int32_t ydtype;
};

__device__ inline int swz(int row, int chunk) { return row * 8 + (chunk ^ (row & 7)); }

template <int B, int TM>
__global__ __launch_bounds__(256, 2) void k_tile_gemm_bf16(TileGemmArgs a, Layout L)
{
    constexpr int MB = TM / 32;  // 16-row blocks per wave (two waves along M)
    __shared__ uint4 A_lds[TM * 8];
    __shared__ uint4 B_lds[kTN * 8];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, r = lane & 15, g = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = int64_t(blockIdx.y) * TM, n0 = int64_t(blockIdx.x) * kTN;

    // decode duty of this wave: strips sid[0], sid[1] of the workgroup's eight
    const DirEntry *dir = reinterpret_cast<const DirEntry *>(a.blob + L.dir_off);
    int64_t sid[2];
    const uint8_t *tile[2] = {nullptr, nullptr};
    TileStreams ts[2] = {};
    uint32_t ru[2] = {0, 0}, rd[2] = {0, 0};
#pragma unroll
    for (int j = 0; j < 2; ++j) sid[j] = n0 / kStripRows + 2 * wave + j;

    f32x4 acc[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[mb][s] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int arow = tid >> 3, achunk = tid & 7;  // A loader: rows arow + 32 i, one 16-byte chunk

    for (int64_t kp = 0; kp < L.KP; ++kp) {
        const int p = int(kp & 7);
        const int64_t kt = kp >> 3;
        // ---- global loads of the A tile (issued first: longest latency)
        uint4 areg[TM / 32];
        const int64_t k = kp * kPanelK + achunk * 8;
#pragma unroll
        for (int i = 0; i < TM / 32; ++i) {
            const int64_t m = m0 + arow + 32 * i;
            areg[i] = make_uint4(0, 0, 0, 0);
            if (m < a.M && k + 8 <= L.K) areg[i] = *reinterpret_cast<const uint4 *>(a.X + m * a.ldx + k);
        }
        // ---- decode this wave's two strip-panels into the B tile
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (sid[j] < L.NS) {
                if (p == 0) {
                    const DirEntry de = dir[sid[j] * L.KT + kt];
                    tile[j] = a.blob + L.streams_off + uint64_t(de.off16) * 16;
                    ts[j] = tile_streams(B, 2, kTilePanels, de.nU, de.nD);
                    ru[j] = 0;
                    rd[j] = 0;
                }
                decode_panel_bf16<B>(tile[j], ts[j], p, ru[j], rd[j], lane, w);
            }
            const int row = (2 * wave + j) * 16 + r;
            B_lds[swz(row, 2 * g)] = make_uint4(w[0], w[1], w[2], w[3]);
            B_lds[swz(row, 2 * g + 1)] = make_uint4(w[4], w[5], w[6], w[7]);
        }
#pragma unroll
        for (int i = 0; i < TM / 32; ++i) A_lds[swz(arow + 32 * i, achunk)] = areg[i];
        __syncthreads();
        // ---- MFMA over the 64 k of the panel
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint4 bf[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) bf[s] = B_lds[swz(wn * 64 + s * 16 + r, 2 * g + h)];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const uint4 af = A_lds[swz(wm * (TM / 2) + mb * 16 + r, 2 * g + h)];
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc[mb][s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, af), __builtin_bit_cast(bf16x8, bf[s]), acc[mb][s], 0, 0, 0);
            }
        }
        __syncthreads();
    }
    // ---- epilogue: lane holds Y[m = 4 g + v][n = r] of each 16 x 16 block
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int64_t n = n0 + wn * 64 + s * 16 + r;
            if (n >= L.N) continue;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t m = m0 + wm * (TM / 2) + mb * 16 + 4 * g + v;
                if (m >= a.M) continue;
                if (a.ydtype == MUW_F32)
                    static_cast<float *>(a.Y)[m * a.ldy + n] = acc[mb][s][v];
                else
                    static_cast<uint16_t *>(a.Y)[m * a.ldy + n] = f32_to_bf16_rne(acc[mb][s][v]);
            }
        }
}

template <int B>
muw_status launch_tile_b(const TileGemmArgs &a, const Layout &L, hipStream_t st)
{
    const unsigned nt = unsigned((L.N + kTN - 1) / kTN);
    if (a.M > 128) {
        dim3 grid(nt, unsigned((a.M + 255) / 256));
        k_tile_gemm_bf16<B, 256><<<grid, 256, 0, st>>>(a, L);
    } else {
        dim3 grid(nt, unsigned((a.M + 127) / 128));
        k_tile_gemm_bf16<B, 128><<<grid, 256, 0, st>>>(a, L);
    }
    return hip_status(hipGetLastError());
}

}  // namespace

bool tile_gemm_applicable(const muw_desc &d, const Layout &L, const GemmArgs &a)
{
    if (d.wdtype != MUW_BF16 || a.blobs || a.M <= 16) return false;
    if (L.K % 8 != 0 || a.ldx % 8 != 0 || (reinterpret_cast<uintptr_t>(a.X) & 15u)) return false;
    if ((a.M + 127) / 128 > 65535) return false;
    return true;
}

muw_status launch_tile_gemm(const muw_desc &d, const Layout &L, const GemmArgs &g, hipStream_t st)
{
    TileGemmArgs a{static_cast<const uint8_t *>(g.blob), static_cast<const uint16_t *>(g.X), g.Y, g.M, g.ldx,
                   g.ldy, g.ydtype};
    switch (d.B) {
    case 4: return launch_tile_b<4>(a, L, st);
    case 8: return launch_tile_b<8>(a, L, st);
    case 16: return launch_tile_b<16>(a, L, st);
    default: return MUW_EUNSUPPORTED;
    }
}

}  // namespace muw
