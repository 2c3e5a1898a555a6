// astraea_sparse_linear, bf16: a per-token linear layer evaluated for the selected tokens only
// (paper, Algorithm 1: Q = X_in[I_sel] W_Q; Sec. 3.2: every layer that acts on a token by itself is
// computed for the selected tokens and reused from the cache for the others; FLOPs appendix: the
// projection and MLP terms):
//     y[row_out(r), o] = act( sum_c x[row_in(r), c] * w[o, c] + bias[o] )
// Rows are gathered by index while the input tile is copied into LDS and scattered by index in the
// epilogue, so neither a compact copy of the input nor one of the output exists.
//
// Shape of the computation on gfx950:
//  * x rows and w rows are both contiguous along the contraction, which is what both operands of
//    v_mfma_f32_32x32x16_bf16 want (a lane holds 8 consecutive k of one row / column).  w feeds the A
//    operand and x the B operand, so that an accumulator lane owns one token and 4 consecutive output
//    features per register group: the epilogue packs them to 8-byte stores along the output row.
//  * workgroup = 8 waves, two per SIMD, output tile 256 features x 256 tokens, each wave 128 features
//    x 64 tokens (4 x 2 MFMA blocks, 128 accumulator registers, 3 LDS fragment reads per 4 MFMAs).
//    One wave per SIMD with 128 x 128 (kWaves = 4, every wave copying, the step's barrier moved in
//    front of the last quarter so that no fragment read follows it) runs fewer clocks per step at a
//    lower clock rate, or the other way round: the chip holds its power limit and the two designs
//    end up within 1 % of each other.
//  * the contraction advances in steps of 64; the two 32 KiB tiles of a step go from global memory
//    straight into LDS (global_load_lds_dwordx4, per-lane addresses, so the row gather costs nothing),
//    double buffered, 16-byte chunks XOR-swizzled inside each 128-byte row against bank conflicts.
//    A copy must cover whole 128-byte lines: with 64-byte pieces (a ring of four 32-deep units) the
//    L1 fetches every line from L2 twice and the kernel is 30 % slower.
//    The second wave of each SIMD issues the copy instructions of the next step, one behind each of
//    its first 16 MFMAs, and has the higher priority: the memory pipe holds it at every copy, and its
//    neighbour's MFMAs fill exactly that time.  A 4-byte load per row touches the lines of two
//    steps ahead so that the copies hit in L2.
//  * workgroup ids are mapped so that the 32 workgroups resident on one XCD form an 8 x 4 block of
//    tiles: they stream 8 row tiles and 4 weight tiles through that XCD's L2 instead of 32 + 32.
#include "gfx950.h"

namespace astraea {
namespace {


constexpr int kBm = 256;                 // tokens per tile
constexpr int kBn = 256;                 // output features per tile
constexpr int kBk = 64;                  // contraction step
constexpr int kRowBytes = kBk * 2;       // 128 B of a row per step
constexpr int kTileBytes = 256 * kRowBytes;          // 32 KiB
constexpr int kStageBytes = 2 * kTileBytes;          // w tile, then x tile
constexpr int kWaves = 8;                // two per SIMD, 128 features x 64 tokens each
constexpr int kTb = 16 / kWaves;         // 32-token MFMA blocks per wave
constexpr int kCopyWaves = kWaves / 2;   // the waves that issue the tile copies (the second wave of each SIMD)
constexpr int kCopies = 32 / kCopyWaves; // 1 KiB copy instructions per copying wave and tile
constexpr int kNumXcd = 8;
constexpr int kSbM = 8, kSbN = 4;        // tiles of one XCD round: 8 token tiles x 4 feature tiles

// Waits until only the two most recent vector-memory instructions (the L2 warm-up loads) are pending:
// the counter retires loads in order, so everything issued before them has then landed.
__device__ __forceinline__ void wait_dma_keep2() { asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); }
// A 4-byte load per lane whose only purpose is to pull its 128-byte line into L2.  It is the copy form
// of the load (global -> LDS), aimed at a 256-byte scrap area every wave may scribble on: the data lands
// whenever it arrives, and with no register as its destination nothing the compiler does with registers
// in the meantime can be hit by it.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"    // m0 is a reserved register; naming it as clobbered is the point
__device__ __forceinline__ void touch_line(const void *gbase, uint32_t goff, uint32_t lds_scrap)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(lds_scrap), "v"(goff), "s"(gbase)
                 : "memory", "m0");
}
#pragma clang diagnostic pop

// Nothing moves across it: the order of MFMAs, fragment reads and copies inside a step is the written one.
#define SB() __builtin_amdgcn_sched_barrier(0)

struct LinearArgs {
    const __bf16 *x;
    const __bf16 *w;
    const __bf16 *bias;        // or null
    __bf16 *y;
    const int32_t *idx_sel;    // or null when neither side is indexed
    int64_t ldx, ldy;          // row strides in elements
    int32_t k_sel, c_in, c_out;
    int32_t n_rows;            // rows of the indexed buffer(s): indices outside [0, n_rows) read a valid row, write none
    int32_t x_indexed, y_indexed, act;
    int32_t m_tiles, n_tiles, sb_n;   // tile counts and 4-wide super-block count along the features
};

__global__ __launch_bounds__(kWaves *kWave, 1) void linear_bf16_kernel(LinearArgs a)
{
    // [stage][w tile | x tile].  Stage flips XOR offsets relative to this array, never absolute addresses.
    constexpr int kPitch = 272;          // epilogue staging: 128 features of a token, padded
    constexpr int kEpiBytes = kWaves * 64 * kPitch;   // every wave stages 64 tokens at a time
    __shared__ __attribute__((aligned(1024))) char lds[2 * kStageBytes > kEpiBytes ? 2 * kStageBytes : kEpiBytes];
    __shared__ __attribute__((aligned(256))) uint32_t scrap[kWave];      // where the L2 warm-up loads land
    // destination rows and bias of this tile, fetched while the first step's tiles are on their way: the
    // epilogue then reads them from LDS instead of waiting for global loads three times over
    __shared__ int32_t tile_rows[kBm];
    __shared__ __attribute__((aligned(16))) uint16_t tile_bias[kBn];

    // ---- which tile: workgroup ids reach the XCDs round-robin; each XCD takes every 8th super-block
    // of 8 x 4 tiles and runs its 32 tiles at the same time.
    const int xcd = blockIdx.x % kNumXcd, seq = blockIdx.x / kNumXcd;
    const int sb = (seq / (kSbM * kSbN)) * kNumXcd + xcd, inner = seq % (kSbM * kSbN);
    const int mt = (sb / a.sb_n) * kSbM + inner % kSbM;
    const int nt = (sb % a.sb_n) * kSbN + inner / kSbM;
    if (mt >= a.m_tiles || nt >= a.n_tiles) return;
    const int m0 = mt * kBm, n0 = nt * kBn;

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int qc = lane & 31, hf = lane >> 5;
    const int wn = wave & 1, wm = wave >> 1;          // this wave's 128 features and 32*kTb tokens of the tile
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    // thread t < 256: destination row of the tile's token t (-1: not stored) and bias of its feature t
    int32_t my_row = -1;
    uint16_t my_bias = 0;
    if (tid < kBm) {
        const int m = m0 + tid;
        if (m < a.k_sel) {
            my_row = m;
            if (a.y_indexed) {
                const int32_t ix = a.idx_sel[m];
                my_row = (uint32_t)ix < (uint32_t)a.n_rows ? ix : -1;
            }
        }
        const int n = n0 + tid;
        if (a.bias && n < a.c_out) my_bias = reinterpret_cast<const uint16_t *>(a.bias)[n];
    }

    // ---- tile copies.  The memory pipe accepts a 1 KiB copy instruction only every ~16 clocks per CU
    // (~57 per wave with four waves at it), so the 64 of a step hold whoever issues them for half a step.
    // The second wave of each SIMD does all of it, one copy behind each of its first 16 MFMAs, and runs at
    // the higher priority: while it is held at a copy the first wave's MFMAs have the matrix pipe, and
    // when it is not, its own go first.  Both waves end their step at about the same time.
    // One instruction fills 8 rows of a tile; copying wave c = wave - 4 issues instructions c, c+4, ...,
    // c+28 of each tile.  Lane l serves row 8*i + l/8 and the physical chunk l%8, which holds logical
    // chunk (l%8) ^ ((row/2)%8); for the rows of one wave that is the same in all 8 instructions, so a
    // lane's byte offset inside its rows is fixed.
    const bool copier = wave >= kCopyWaves;
    const int cw = wave & (kCopyWaves - 1);
    if (copier) __builtin_amdgcn_s_setprio(1);
    const int d_row = lane >> 3;
    const int lchunk = (lane & 7) ^ ((4 * (cw & 1) + (lane >> 4)) & 7);
    uint32_t woff[kCopies], xoff[kCopies];   // byte offsets of this lane's rows from w and x
#pragma unroll
    for (int t = 0; t < kCopies; ++t) {
        const int r = 8 * (cw + kCopyWaves * t) + d_row;
        int n = n0 + r;                  // rows past the end re-read the last one; they are never stored
        if (n > a.c_out - 1) n = a.c_out - 1;
        woff[t] = (uint32_t)n * (uint32_t)a.c_in * 2u + (uint32_t)lchunk * 16u;
        int m = m0 + r;
        if (m > a.k_sel - 1) m = a.k_sel - 1;
        const int64_t row = a.x_indexed ? (int64_t)clamp_row(a.idx_sel[m], a.n_rows) : (int64_t)m;
        xoff[t] = (uint32_t)(row * a.ldx * 2) + (uint32_t)lchunk * 16u;
    }
    // all index loads must have landed before the loop: a load still pending at the loop header would
    // make the compiler wait on the vector-memory counter inside it
#pragma unroll
    for (int t = 0; t < kCopies; ++t) asm volatile("" ::"v"(xoff[t]), "v"(woff[t]));

    const char *wg = reinterpret_cast<const char *>(a.w);
    const char *xg = reinterpret_cast<const char *>(a.x);
    // L2 warm-up: a step's 128 bytes of one row are one cache line, and this wave copies 64 rows of
    // each tile, so one lane per row touches all of them (lane l: the l/8-th copy's row l%8).
    // Rows come from HBM (gathered x rows) or the memory-side cache (w), whose latency exceeds one step;
    // touching them kPrefetch steps ahead lets the tile copies hit in L2.
    uint32_t pf_w, pf_x;
    {
        const int r = 8 * (cw + kCopyWaves * ((lane >> 3) % kCopies)) + (lane & 7);
        int n = n0 + r;
        if (n > a.c_out - 1) n = a.c_out - 1;
        pf_w = (uint32_t)n * (uint32_t)a.c_in * 2u;
        int m = m0 + r;
        if (m > a.k_sel - 1) m = a.k_sel - 1;
        const int64_t row = a.x_indexed ? (int64_t)clamp_row(a.idx_sel[m], a.n_rows) : (int64_t)m;
        pf_x = (uint32_t)(row * a.ldx * 2);
    }
    asm volatile("" ::"v"(pf_x), "v"(pf_w));
    const uint32_t scrap0 = (uint32_t)(uintptr_t)scrap;
    constexpr int kPrefetch = 2;      // 3: 2-3 % slower, 1: the copy is already on its way
    auto dma_w = [&](int t, int kstep, uint32_t stage) __attribute__((always_inline)) {
        dma16(wg + (int64_t)kstep * kRowBytes, woff[t], lds0 + stage + (cw + kCopyWaves * t) * 1024);
    };
    auto dma_x = [&](int t, int kstep, uint32_t stage) __attribute__((always_inline)) {
        dma16(xg + (int64_t)kstep * kRowBytes, xoff[t], lds0 + stage + kTileBytes + (cw + kCopyWaves * t) * 1024);
    };

    // ---- fragment offsets inside the array: row 32*block + qc of this wave's half, logical chunk 2*s + hf of k-step s
    uint32_t wa[4], xa[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const uint32_t sw = (uint32_t)(((2 * s + hf) ^ ((qc >> 1) & 7)) << 4);
        wa[s] = (wn * 128 + qc) * kRowBytes + sw;
        xa[s] = kTileBytes + (wm * 32 * kTb + qc) * kRowBytes + sw;
    }

    floatx16 acc[4][kTb];                // [feature block][token block]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < kTb; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    const int nk = a.c_in / kBk;
    // prologue: first stage
    if (copier) {
#pragma unroll
        for (int t = 0; t < kCopies; ++t) {
            dma_w(t, 0, 0);
            dma_x(t, 0, 0);
        }
        for (int p = 1; p < kPrefetch; ++p) {
            const int kp = p < nk ? p : nk - 1;
            touch_line(wg + (int64_t)kp * kRowBytes, pf_w, scrap0);
            touch_line(xg + (int64_t)kp * kRowBytes, pf_x, scrap0);
        }
    }
    wait_dma();
    if (tid < kBm) {
        tile_rows[tid] = my_row;
        tile_bias[tid] = my_bias;
    }
    __builtin_amdgcn_s_barrier();

    bf16x8 wf[2][4], xf[2][kTb];
    // the fragments of a step's first quarter
    auto read_first = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kTb; ++j) xf[0][j] = lds_read_b128(lds0 + xa[0] + j * 32 * kRowBytes);
#pragma unroll
        for (int i = 0; i < 4; ++i) wf[0][i] = lds_read_b128(lds0 + wa[0] + i * 32 * kRowBytes);
    };
    uint32_t next_stage = kStageBytes;   // where the copies of step kk+1 go
    int kn = 0, kp = 0;
    // Quarter s of a step, in the order written: behind each of its first MFMAs one fragment read of quarter
    // s + 1; a copying wave also puts one tile copy behind each MFMA of quarters 0 and 1 and the two warm-up
    // loads into quarter 2.  The memory pipe takes a copy every ~16 clocks per CU, ~57 per wave with four
    // waves at it, so a copying wave spends half a step held up at its copies; its SIMD neighbour's MFMAs
    // run in exactly that time.
    auto quarter = [&](auto s_tag) __attribute__((always_inline)) {
        constexpr int s = decltype(s_tag)::value;
        constexpr int cur = s & 1, nxt = cur ^ 1;
#pragma unroll
        for (int n = 0; n < 4 * kTb; ++n) {
            const int i = n / kTb, j = n % kTb;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][i], xf[cur][j], acc[i][j], 0, 0, 0);
            if (s < 3) {
                if (n < kTb) xf[nxt][n] = lds_read_b128(lds0 + xa[(s + 1) & 3] + n * 32 * kRowBytes);
                else if (n < kTb + 4) wf[nxt][n - kTb] = lds_read_b128(lds0 + wa[(s + 1) & 3] + (n - kTb) * 32 * kRowBytes);
            }
            if (s < 2) {
                const int c = s * 4 * kTb + n;          // 0 .. 15
                if (copier) {
                    if (c & 1) dma_x(c >> 1, kn, next_stage);
                    else dma_w(c >> 1, kn, next_stage);
                }
            } else if (s == 2 && n < 2) {
                if (copier) {
                    if (n == 0) touch_line(wg + (int64_t)kp * kRowBytes, pf_w, scrap0);
                    else touch_line(xg + (int64_t)kp * kRowBytes, pf_x, scrap0);
                }
            }
            SB();
        }
    };
    using Q0 = std::integral_constant<int, 0>;
    using Q1 = std::integral_constant<int, 1>;
    using Q2 = std::integral_constant<int, 2>;
    using Q3 = std::integral_constant<int, 3>;
    for (int kk = 0; kk < nk; ++kk) {
        // the last step has nothing to prefetch: it copies its own tiles again into the idle stage
        // rather than branch around every copy
        kn = kk + 1 < nk ? kk + 1 : kk;
        kp = kk + kPrefetch < nk ? kk + kPrefetch : nk - 1;
        read_first();
        SB();
        quarter(Q0{});
        quarter(Q1{});
        quarter(Q2{});
        quarter(Q3{});
        // the next step's tiles are complete and this step's are no longer read: swap stages
        wait_dma_keep2();
        __builtin_amdgcn_s_barrier();
        SB();
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            wa[s] ^= kStageBytes;
            xa[s] ^= kStageBytes;
        }
        next_stage ^= kStageBytes;
    }

    wait_dma();
    // ---- epilogue: bias, activation, bf16; then through LDS so that global stores cover whole rows.
    // Register group g of block (i, j): features 128*wn + 32*i + 8*g + 4*hf + 0..3, token
    // 32*kTb*wm + 32*j + qc of the tile.  An accumulator lane owns one token, so stores straight from the
    // registers would put 16 bytes on each of 32 rows per instruction; partial-line writes of that kind
    // cost several times the main loop's share of HBM time.  Instead each wave transposes its block,
    // 64 tokens at a time, through its own 17 KiB of LDS (rows of 128 features, pitch 272
    // bytes) and writes 4 rows x 256 contiguous bytes per instruction.  The tile buffers are free: every
    // wave has passed the barrier that ends the last step.  The region is private to the wave, so no
    // workgroup barrier is needed, only the wave's own LDS counter.
    // this lane's 64 bias values (16 groups of 4 features), from the copy in LDS
    uint2v bias2[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g)
            bias2[i][g] = *reinterpret_cast<const uint2v *>(&tile_bias[wn * 128 + 32 * i + 8 * g + 4 * hf]);
    const uint32_t ebase = lds0 + wave * (64 * kPitch);
    const int o_row = lane >> 4, o_chunk = lane & 15;      // read-back: 4 rows per instruction, 16 lanes x 16 B each
#pragma unroll
    for (int jh = 0; jh < kTb / 2; ++jh) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int j = 2 * jh + jj;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int nl = 32 * i + 8 * g + 4 * hf;      // feature inside the wave's 128
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * g + e];
                    const uint2v b2 = bias2[i][g];
                    v[0] += __uint_as_float(b2[0] << 16);
                    v[1] += __uint_as_float(b2[0] & 0xffff0000u);
                    v[2] += __uint_as_float(b2[1] << 16);
                    v[3] += __uint_as_float(b2[1] & 0xffff0000u);
                    if (a.act == ASTRAEA_ACT_GELU_TANH) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = gelu_tanh(v[e]);
                    }
                    uint2v o2;
                    o2[0] = pack_bf16(v[0], v[1]);
                    o2[1] = pack_bf16(v[2], v[3]);
                    *reinterpret_cast<uint2v __attribute__((address_space(3))) *>(
                        (uintptr_t)(ebase + (32 * jj + qc) * kPitch + nl * 2)) = o2;
                }
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);                      // lgkmcnt(0): this wave's LDS writes are done
        // destination rows of this half first (16 per lane), then the stores: an index load between
        // two stores would be waited for each time
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int tl = 4 * it + o_row;                       // token inside this half
            const int64_t orow = tile_rows[wm * 32 * kTb + 64 * jh + tl];    // -1: past the end or a bad index
            const int n = n0 + wn * 128 + 8 * o_chunk;           // c_out is a multiple of 8: a chunk is all in or all out
            const uint4v val = *reinterpret_cast<const uint4v __attribute__((address_space(3))) *>(
                (uintptr_t)(ebase + tl * kPitch + o_chunk * 16));
            // written once: streaming stores leave the tiles other workgroups still read in L2 (+1-3 %)
            if (n < a.c_out && orow >= 0)
                __builtin_nontemporal_store(val, reinterpret_cast<uint4v *>(a.y + orow * a.ldy + n));
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);                      // reads done before the second half overwrites
    }
}


}  // namespace

int launch_linear_bf16(const void *x, const void *w, const void *bias, void *y, const int32_t *idx_sel, int64_t k_sel,
                       int64_t n_rows, int32_t c_in, int32_t c_out, int64_t ldx, int64_t ldy, int x_indexed, int y_indexed, int act,
                       hipStream_t stream)
{
    if (k_sel == 0) return ASTRAEA_OK;
    LinearArgs a;
    a.x = (const __bf16 *)x;
    a.w = (const __bf16 *)w;
    a.bias = (const __bf16 *)bias;
    a.y = (__bf16 *)y;
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
    a.m_tiles = (int32_t)((k_sel + kBm - 1) / kBm);
    a.n_tiles = (c_out + kBn - 1) / kBn;
    a.sb_n = (a.n_tiles + kSbN - 1) / kSbN;
    const int64_t sb_m = (a.m_tiles + kSbM - 1) / kSbM;
    const int64_t sbs = sb_m * a.sb_n;                                  // super-blocks, dealt round-robin to the XCDs
    const int64_t rounds = (sbs + kNumXcd - 1) / kNumXcd;
    const int64_t grid = rounds * kNumXcd * (kSbM * kSbN);
    if (grid > 2147483647LL) return fail(ASTRAEA_ERR_INVALID, "astraea_sparse_linear: grid too large");
    hipLaunchKernelGGL(linear_bf16_kernel, dim3((unsigned)grid), dim3(kWaves * kWave), 0, stream, a);
    return check_launch("astraea_sparse_linear(bf16)");
}

}  // namespace astraea
