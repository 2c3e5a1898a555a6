// astraea_sparse_linear, fp32 mode: y[row_out(r), :] = act(x[row_in(r), :] W^T + b) for the selected
// rows only (paper, Algorithm 1 steps 4-5, "Q = X_in[I_sel] W_Q", and in the same way every projection
// and MLP layer of a block; FLOPs appendix, the 2*N*D*D' terms with N -> number of selected tokens).
//
// The accuracy-first twin of the bf16 kernel, for the fp32 configuration: everything stays in fp32 on
// v_mfma_f32_32x32x2_f32.  x rows and W rows are both contiguous along the contraction, so W feeds the
// A operand and x the B operand (the transposed form, as in the bf16 kernel): a lane owns one token
// and, per accumulator block, 16 features in groups of 4 consecutive ones, which it stores as 16 bytes.
// No LDS: lane (r = l % 32, hf = l / 32) reads, for a step of 16 contraction indices, the 8 floats
// k0 + 8*hf .. k0 + 8*hf + 7 of row r of each operand block (two 16-byte loads) and MFMA j of the step
// contracts indices {k0 + j, k0 + 8 + j}; the next step's loads are in flight during the MFMAs.
// Workgroup = 4 waves in a 2 x 2 arrangement, 128 features x 128 tokens; a wave 64 x 64.
//
// MFMA-bound in principle (157.3 TFLOP/s fp32), in practice bound by the operand loads: each wave
// re-reads its 64 + 64 rows from L2 (16 flops per byte).  It serves the small fp32 layers; the bf16
// kernel carries the throughput.
#include "gfx950.h"

namespace astraea {
namespace {


constexpr int kWaves = 4;
constexpr int kTile = 128;          // features and tokens per workgroup
constexpr int kStep = 16;           // contraction indices per step

struct LinearF32Args {
    const float *x;
    const float *w;
    const float *bias;         // or null
    float *y;
    const int32_t *idx_sel;    // or null when neither side is indexed
    int64_t ldx, ldy;          // row strides in elements
    int32_t k_sel, c_in, c_out;
    int32_t n_rows;            // rows of the indexed buffer(s): indices outside [0, n_rows) read a valid row, write none
    int32_t x_indexed, y_indexed, act;
    int32_t n_tiles;           // feature tiles; workgroup id = token tile * n_tiles + feature tile
};

struct Frag {
    float4 lo, hi;             // contraction indices 8*hf + 0..3 and 8*hf + 4..7 of this lane's row
};

__device__ __forceinline__ Frag load_frag(const float *row, int k0)
{
    Frag f;
    f.lo = *reinterpret_cast<const float4 *>(row + k0);
    f.hi = *reinterpret_cast<const float4 *>(row + k0 + 4);
    return f;
}
__device__ __forceinline__ float frag_at(const Frag &f, int j)
{
    switch (j) {
    case 0: return f.lo.x;
    case 1: return f.lo.y;
    case 2: return f.lo.z;
    case 3: return f.lo.w;
    case 4: return f.hi.x;
    case 5: return f.hi.y;
    case 6: return f.hi.z;
    default: return f.hi.w;
    }
}

__global__ __launch_bounds__(kWaves *kWave) void linear_f32_kernel(LinearF32Args a)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int r = lane & 31, hf = lane >> 5;
    const int wn = wave & 1, wm = wave >> 1;
    const int tile_n = blockIdx.x % a.n_tiles, tile_m = blockIdx.x / a.n_tiles;
    const int n0 = tile_n * kTile + wn * 64;           // first feature of this wave
    const int m0 = tile_m * kTile + wm * 64;           // first selected row of this wave

    // this lane's rows of the two feature blocks (A) and the two token blocks (B); rows past the end
    // re-read the last valid one and are never stored
    const float *wrow[2];
    const float *xrow[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        int n = n0 + 32 * b + r;
        if (n > a.c_out - 1) n = a.c_out - 1;
        wrow[b] = a.w + (int64_t)n * a.c_in + 8 * hf;
        int m = m0 + 32 * b + r;
        if (m > a.k_sel - 1) m = a.k_sel - 1;
        const int64_t row = a.x_indexed ? (int64_t)clamp_row(a.idx_sel[m], a.n_rows) : (int64_t)m;
        xrow[b] = a.x + row * a.ldx + 8 * hf;
    }

    floatx16 acc[2][2];        // [feature block][token block]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    Frag wf[2], xf[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        wf[b] = load_frag(wrow[b], 0);
        xf[b] = load_frag(xrow[b], 0);
    }
    for (int k0 = 0; k0 < a.c_in; k0 += kStep) {
        Frag wn_[2], xn_[2];
        const int kn = k0 + kStep < a.c_in ? k0 + kStep : k0;      // the last step re-reads itself, unused
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            wn_[b] = load_frag(wrow[b], kn);
            xn_[b] = load_frag(xrow[b], kn);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x2f32(frag_at(wf[i], j), frag_at(xf[t], j), acc[i][t], 0, 0, 0);
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            wf[b] = wn_[b];
            xf[b] = xn_[b];
        }
    }

    // accumulator register e of block (i, t): feature n0 + 32 i + 8 (e / 4) + 4 hf + e % 4, token m0 + 32 t + r
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int m = m0 + 32 * t + r;
        if (m >= a.k_sel) continue;
        int64_t orow = m;
        if (a.y_indexed) {
            const int32_t ix = a.idx_sel[m];
            if ((uint32_t)ix >= (uint32_t)a.n_rows) continue;       // a row index outside the buffer writes nothing
            orow = ix;
        }
        float *yp = a.y + orow * a.ldy;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + 32 * i + 8 * g + 4 * hf;         // c_out is a multiple of 8: all four in or all out
                if (n >= a.c_out) continue;
                float4 v = make_float4(acc[i][t][4 * g], acc[i][t][4 * g + 1], acc[i][t][4 * g + 2], acc[i][t][4 * g + 3]);
                if (a.bias) {
                    const float4 b4 = *reinterpret_cast<const float4 *>(a.bias + n);
                    v.x += b4.x;
                    v.y += b4.y;
                    v.z += b4.z;
                    v.w += b4.w;
                }
                if (a.act == ASTRAEA_ACT_GELU_TANH) {
                    v.x = gelu_tanh(v.x);
                    v.y = gelu_tanh(v.y);
                    v.z = gelu_tanh(v.z);
                    v.w = gelu_tanh(v.w);
                }
                *reinterpret_cast<float4 *>(yp + n) = v;
            }
    }
}

}  // namespace

int launch_linear_f32(const void *x, const void *w, const void *bias, void *y, const int32_t *idx_sel, int64_t k_sel,
                      int64_t n_rows, int32_t c_in, int32_t c_out, int64_t ldx, int64_t ldy, int x_indexed,
                      int y_indexed, int act, hipStream_t stream)
{
    if (k_sel == 0) return ASTRAEA_OK;
    LinearF32Args a;
    a.x = (const float *)x;
    a.w = (const float *)w;
    a.bias = (const float *)bias;
    a.y = (float *)y;
    a.idx_sel = idx_sel;
    a.ldx = ldx;
    a.ldy = ldy;
    a.k_sel = (int32_t)k_sel;
    a.n_rows = (int32_t)n_rows;
    a.c_in = c_in;
    a.c_out = c_out;
    a.x_indexed = x_indexed;
    a.y_indexed = y_indexed;
    a.act = act;
    const int64_t gx = (c_out + kTile - 1) / kTile, gy = (k_sel + kTile - 1) / kTile;
    if (gx * gy > 2147483647LL) return fail(ASTRAEA_ERR_INVALID, "astraea_sparse_linear(fp32): grid too large");
    a.n_tiles = (int32_t)gx;
    hipLaunchKernelGGL(linear_f32_kernel, dim3((unsigned)(gx * gy)), dim3(kWaves * kWave), 0, stream, a);
    return check_launch("astraea_sparse_linear(fp32)");
}

}  // namespace astraea
