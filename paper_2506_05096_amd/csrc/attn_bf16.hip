// astraea_sparse_attn_fwd, bf16 mode, head_dim 128 (paper, Algorithm 1 step 6:
// X_out[I_sel] = Softmax(Q_sel K^T / sqrt(d)) V with every key and value kept, Sec. 3.2
// "Sparse Attention").  Flash-style: K/V are streamed once per query tile, the N x N map is never
// materialised, softmax is the online form in fp32.
//
// Shape of the computation on gfx950:
//  * both products are computed transposed, S^T = K Q^T and O^T = V^T P^T, with
//    v_mfma_f32_32x32x16_bf16.  In every accumulator a lane then owns one query column, so the row
//    max / row sum / rescale factor are per-lane scalars (one exchange between lanes l and l+32),
//    and the S^T accumulator registers, converted to bf16, are the B operand of the second
//    product as they stand: register group 8*(t%2)..+7 of key block t/2 feeds MFMA t, with the key
//    order inside the contraction permuted the same way on the V side.
//  * K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4), double
//    buffered, with no register staging.  Such a load writes 64 x 16 B contiguously, so rows
//    cannot be padded; bank conflicts are avoided by an XOR swizzle of the 16-byte chunks inside
//    each 256-byte row, applied through the per-lane global address.
//  * the LDS pipe issues one wave instruction every ~4.5 clocks whatever its width, so fragments
//    must come in 16-byte reads.  K rows are head-dim contiguous, which is what S^T = K Q^T wants.
//    V is contracted over keys, so a pre-pass rewrites V once per call into 16 KiB tiles of V^T
//    ([128 head-dim rows][64 keys], keys permuted inside each group of 16 to match the register
//    order of P^T, 16-byte chunks already XOR-swizzled); the main kernel then copies a tile
//    linearly into LDS and reads every V^T fragment with one ds_read_b128.  The pre-pass moves
//    2*N*H*D*2 bytes, under 1% of the attention time, and needs N_pad*H*D*2 bytes of workspace.
//  * queries are gathered by index while loading the Q fragment, which then lives in registers
//    for the whole sweep (the "gather" step of the path is fused here).
//  * the exponent offset of a row need not be its exact max: a stale one costs range, not accuracy
//    (P, the row sums and the O accumulators are floating point with 8-bit exponents).  The main
//    kernel therefore fixes each row's offset at the max over the first key tile and takes no max in
//    the sweep at all, which removes a fifth of the softmax arithmetic.  A row whose later logits
//    outgrow that offset by more than 2^80 (or overflow) shows in its final row sum; its workgroup
//    then flags itself, writes nothing, and a second launch of the same kernel in its exact form
//    (a max per tile, lazy rescale when it grew by more than 2^kTau) redoes just the flagged ones.
//  * workgroup ids are mapped so that the workgroups resident on one XCD work on the same head and
//    sweep the keys together; K/V tiles are then served from that XCD's L2.
//  * the two waves that share a SIMD alternate: while one runs the MFMAs of a tile the other runs
//    the exponentials of its own tile, so the matrix pipe and the VALU work at the same time.
#include <type_traits>

#include "gfx950.h"

namespace astraea {
namespace {


constexpr int D = 128;
constexpr int kWaves = 8;
constexpr int kBq = 32 * kWaves;        // queries per workgroup
constexpr int kBk = 64;                 // keys per LDS tile
constexpr int kRowBytes = D * 2;        // 256 B per key row, unpadded
constexpr int kTileBytes = kBk * kRowBytes;          // 16 KiB
constexpr int kBufBytes = 2 * kTileBytes;            // K tile then V tile
constexpr float kTau = 8.0f;            // exact form: lazy-rescale threshold, log2 units
constexpr float kBig = 0x1p80f;         // fast form: a final row sum above this sends the workgroup to the exact form
constexpr int kNumXcd = 8;

__device__ __forceinline__ float xhalf_max(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}



// ---- pre-pass: V [N, H, 128] -> tiles of V^T.  Tile (head, T) is 16 KiB at
// vt + (head * ntiles + T) * 16 KiB and holds keys 64*T .. 64*T+63: row d (128 bytes) = 8 chunks;
// logical chunk c = 2*t + hf holds keys 64*T + 16*t + 8*(j/4) + 4*hf + j%4 for j = 0..7, and is
// stored at physical chunk c ^ ((d >> 1) & 7).  Keys past N are zero.
__global__ __launch_bounds__(256) void transpose_v_kernel(const __bf16 *__restrict__ v, int64_t N, int64_t kv_stride_n,
                                                          int64_t kv_stride_h, int64_t ntiles,
                                                          char *__restrict__ vt)
{
    __shared__ uint16_t tile[kBk][D + 2];      // [key][d], odd dword pitch: column reads conflict-free
    const int64_t T = blockIdx.x;
    const int head = blockIdx.y;
    const uint16_t *vb = reinterpret_cast<const uint16_t *>(v) + (int64_t)head * kv_stride_h;
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (tid >> 4) + 16 * i, c16 = tid & 15;
        const int64_t key = T * kBk + row;
        uint4v val = {0u, 0u, 0u, 0u};
        // V is read once here: streaming hint, the lines are not kept in L2
        if (key < N) val = __builtin_nontemporal_load(reinterpret_cast<const uint4v *>(vb + key * kv_stride_n + c16 * 8));
        uint32_t *dst = reinterpret_cast<uint32_t *>(&tile[row][c16 * 8]);
        dst[0] = val[0];
        dst[1] = val[1];
        dst[2] = val[2];
        dst[3] = val[3];
    }
    __syncthreads();
    char *out = vt + ((int64_t)head * ntiles + T) * kTileBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int o = tid + 256 * i;           // output chunk id: row d = o / 8, logical chunk c = o % 8
        const int d = o >> 3, c = o & 7, t = c >> 1, hf = c & 1;
        uint32_t w[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int j0 = 2 * jj, j1 = 2 * jj + 1;
            const int k0 = 16 * t + 8 * (j0 >> 2) + 4 * hf + (j0 & 3);
            const int k1 = 16 * t + 8 * (j1 >> 2) + 4 * hf + (j1 & 3);
            w[jj] = (uint32_t)tile[k0][d] | ((uint32_t)tile[k1][d] << 16);
        }
        uint4v val = {w[0], w[1], w[2], w[3]};
        *reinterpret_cast<uint4v *>(out + d * 128 + ((c ^ ((d >> 1) & 7)) << 4)) = val;
    }
}

// Budget-aware work split.  Work item = (head, tile of 256 selected queries), head-major; XCD x owns the
// contiguous item range [x * items_per_xcd, (x+1) * items_per_xcd) and workgroups reach XCDs round-robin
// by id.  With 32 CUs per XCD the items of an XCD run in rounds of 32.  The first `full_items` of each
// XCD sweep all keys; the remaining items_per_xcd - full_items (< 32, what would be a mostly idle last
// round) are each cut into `splits` key ranges of `tiles_per_split` tiles, run by as many workgroups,
// whose unnormalised partial results are combined by merge_partials_kernel.  Execution time then
// follows the number of selected tokens instead of the number of rounds.
struct AttnSchedule {
    int64_t items_per_xcd;
    int64_t full_items;
    int64_t tiles_per_split;
    int32_t q_tiles;
    int32_t splits;
};
constexpr int kPartialFloats = kBq * D + 2 * kBq;    // O^T accumulators, then running max, then row sum
constexpr int kMaxSharesPerXcd = 64;

constexpr int MFMA = 0x008, DSR = 0x100;
#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
// Nothing may be moved across a phase boundary: left alone, the scheduler pulls the exponentials next to
// the MFMAs that consume them, i.e. into the other phase.
#define PHASE_BARRIER()                    \
    do {                                   \
        __builtin_amdgcn_sched_barrier(0); \
        __builtin_amdgcn_s_barrier();      \
        __builtin_amdgcn_sched_barrier(0); \
    } while (0)

// EXACT = false: the main launch (offset fixed by the first tile, no max in the sweep); every workgroup
// writes redo[blockIdx.x] = 1 if one of its rows outgrew the offset (and then stores no result), else 0.
// EXACT = true: the second launch over the same grid; a workgroup whose flag is 0 returns at once, the
// others sweep their keys again with a max per tile and store their results.
template <bool EXACT>
__global__ __launch_bounds__(kWaves *kWave, 1) void attn_bf16_kernel(
    const __bf16 *__restrict__ q, const __bf16 *__restrict__ k, const char *__restrict__ vt, int64_t N, int32_t H,
    int64_t q_stride_n, int64_t q_stride_h, int64_t kv_stride_n, int64_t kv_stride_h,
    const int32_t *__restrict__ idx_sel, int64_t k_sel, int q_is_compact, float scale_log2e,
    __bf16 *__restrict__ o_sel, int64_t o_stride_n, int o_scatter, float *__restrict__ lse_sel, AttnSchedule sch,
    float *__restrict__ partial, uint32_t *__restrict__ redo)
{
    // [parity][K tile | V^T tile]; 64 KiB, one 8-wave workgroup per CU (two waves per SIMD)
    __shared__ __attribute__((aligned(1024))) char lds[2 * kBufBytes];
    __shared__ uint32_t wave_outgrew[kWaves];
    if (EXACT && redo && redo[blockIdx.x] == 0) return;     // no flag array: the exact form runs alone

    const int64_t ntiles = (N + kBk - 1) / kBk;
    const int64_t total_items = (int64_t)H * sch.q_tiles;
    const int64_t xcd = blockIdx.x % kNumXcd, slot = blockIdx.x / kNumXcd;
    int64_t item, tile_begin = 0, tile_end = ntiles, pslot = -1;
    if (slot < sch.full_items) {
        item = xcd * sch.items_per_xcd + slot;
    } else {
        const int64_t p = slot - sch.full_items, li = p / sch.splits, sp = p % sch.splits;
        item = xcd * sch.items_per_xcd + sch.full_items + li;
        tile_begin = sp * sch.tiles_per_split;
        tile_end = tile_begin + sch.tiles_per_split < ntiles ? tile_begin + sch.tiles_per_split : ntiles;
        pslot = (xcd * (sch.items_per_xcd - sch.full_items) + li) * sch.splits + sp;
    }
    if (item >= (xcd + 1) * sch.items_per_xcd || item >= total_items) return;
    const int head = (int)(item / sch.q_tiles);
    const int64_t qt = item % sch.q_tiles;

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int qc = lane & 31, hf = lane >> 5;
    const int64_t r0 = qt * kBq + wave * 32;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

    // ---- Q fragment: lane holds query column qc, head-dim 16*s + 8*hf + 0..7 (B operand of K Q^T)
    int64_t r = r0 + qc;
    if (r > k_sel - 1) r = k_sel - 1;               // ragged last tile: duplicate a valid row, never stored
    // an index outside [0, N) reads a valid row instead
    const int64_t qrow = q_is_compact ? r : (int64_t)clamp_row(idx_sel[r], (int32_t)N);
    const __bf16 *qp = q + qrow * q_stride_n + (int64_t)head * q_stride_h + 8 * hf;
    bf16x8 qf[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);

    floatx16 oacc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[b][i] = 0.0f;
    float m_c = -INFINITY;     // running max of scale*log2(e)*logit actually used as exponent offset
    float l_run = 0.0f;        // this lane's share of the running sum

    // ---- tile DMA.  A wave instruction fills 1 KiB of a tile: lane l writes 16 bytes at 16*l.
    // K: block = 4 key rows; physical chunk p of row r holds logical chunk p ^ (r & 15).
    // V^T: the pre-pass already wrote the tile as its LDS image, so the copy is linear.
    const char *kbase = reinterpret_cast<const char *>(k + (int64_t)head * kv_stride_h);
    const char *vtbase = vt + (int64_t)head * ntiles * kTileBytes;
    const int64_t row_pitch = kv_stride_n * 2;       // bytes between consecutive keys
    const int d_row = lane >> 4, d_p = lane & 15;
    const uint32_t lin_off = lane * 16;
    // Copies one tile with NW waves taking part (this wave is number w of them): block b of the
    // tile is copied by wave b % NW.
    auto dma_v_tile = [&](int64_t tile, int par, int w, auto nw_tag) __attribute__((always_inline)) {
        constexpr int NW = decltype(nw_tag)::value;
        const char *src = vtbase + tile * kTileBytes + w * 1024;
        const uint32_t dst = lds0 + par * kBufBytes + kTileBytes + w * 1024;
#pragma unroll
        for (int i = 0; i < 16 / NW; ++i) dma16(src + i * NW * 1024, lin_off, dst + i * NW * 1024);
    };
    auto dma_k_tile = [&](int64_t tile, int par, int w, auto nw_tag) __attribute__((always_inline)) {
        constexpr int NW = decltype(nw_tag)::value;  // 4 or 8: a wave's rows advance by 16 or 32 per step,
        const int64_t key0 = tile * kBk;             // so row & 15 (the swizzle) is the same for all of them
        const char *src = kbase + key0 * row_pitch;
        const uint32_t dst = lds0 + par * kBufBytes + w * 1024;
        const int row0 = 4 * w + d_row;
        const uint32_t sw = (uint32_t)((d_p ^ (row0 & 15)) << 4);
        if (key0 + kBk <= N) {
            const uint32_t off = (uint32_t)row0 * (uint32_t)row_pitch + sw;
#pragma unroll
            for (int i = 0; i < 16 / NW; ++i) dma16(src + i * 4 * NW * row_pitch, off, dst + i * NW * 1024);
        } else {
            const int64_t last = N - 1 - key0;       // rows past the last key re-read it (masked later)
#pragma unroll
            for (int i = 0; i < 16 / NW; ++i) {
                const int rr = row0 + 4 * NW * i;
                const int64_t rc = rr < last ? rr : last;
                dma16(src, (uint32_t)(rc * row_pitch) + sw, dst + i * NW * 1024);
            }
        }
    };

    // ---- LDS read offsets relative to a buffer pair; the buffer parity and the array's base are added where
    // the offsets are used (the tile loop is unrolled by two, so the parity is a compile-time constant there
    // and lands in the read's immediate offset)
    // K fragment (kb, s): row 32*kb + qc, logical chunk 2*s + hf; kb is an immediate offset
    uint32_t ka[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) ka[s] = qc * kRowBytes + (((2 * s + hf) ^ (qc & 15)) << 4);
    // V^T fragment (tt, b): row d = 32*b + qc (128-byte rows), logical chunk 2*tt + hf; b is an immediate
    uint32_t va[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
        va[tt] = kTileBytes + qc * 128 + (((2 * tt + hf) ^ ((qc >> 1) & 7)) << 4);

    floatx16 sacc[2];          // S^T of the current tile (two blocks of 32 keys)
    uint32_t pw[16];           // P^T as bf16 pairs: pw[8*kb + i] = registers 2i, 2i+1 of block kb

    // VALU phase for tile j: exponentials -> pw, row sums; in the exact form first the row max: the running
    // max is only raised (and what was accumulated under the old one rescaled) when some row's max moved up by
    // more than 2^kTau, otherwise the stale max stays in use.
    // register i of sacc[kb]: key = 64*j + 32*kb + (i/4)*8 + hf*4 + i%4, query = qc
    auto tile_row_max = [&]() __attribute__((always_inline)) -> float {
        float tm = sacc[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) tm = fmaxf(tm, sacc[kb][i]);
        return xhalf_max(tm) * scale_log2e;
    };
    auto softmax_tile = [&](int64_t j) __attribute__((always_inline)) {
        if ((j + 1) * kBk > N) {                    // only the last tile can be ragged
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = (int)(j * kBk - N) + 32 * kb + (i >> 2) * 8 + hf * 4 + (i & 3);
                    if (key >= 0) sacc[kb][i] = -INFINITY;
                }
        }
        if (EXACT) {
            const float tmax = tile_row_max();
            if (__builtin_amdgcn_ballot_w64(tmax > m_c + kTau) != 0) {
                const float m_new = fmaxf(m_c, tmax);
                const float alpha = __builtin_amdgcn_exp2f(m_c - m_new);   // 0 on the first tile
                m_c = m_new;
                l_run *= alpha;
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;
            }
        }
        float ps0 = 0.0f, ps1 = 0.0f;
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int kb = u >> 3, i = 2 * (u & 7);
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][i], scale_log2e, -m_c));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][i + 1], scale_log2e, -m_c));
            pw[u] = pack_bf16(p0, p1);
            // the row sum adds the rounded values, the same ones the second product uses
            if (u & 1)
                ps1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[u]), ones, ps1, false);
            else
                ps0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pw[u]), ones, ps0, false);
        }
        l_run += ps0 + ps1;
        // keep the row-sum arithmetic in this phase (it is not needed until the end of the sweep, and
        // would otherwise drift behind the MFMAs of the next phase)
        asm volatile("" : "+v"(l_run));
    };

    constexpr int kAhead = 4;      // an MFMA's fragment is fetched kAhead MFMAs before it issues
    // MFMA phase.  O^T += V^T(j) P^T(j): 16 MFMAs; group tt contracts the 16 keys 16*tt + {0..3, 8..11}
    // (lanes 0-31) and 16*tt + {4..7, 12..15} (lanes 32-63); V^T(j) is in the parity va[] points at.
    // Then, if WITH_QK, S^T = K Q^T for the next tile: 16 MFMAs, the two blocks of 32 keys taking turns (two
    // consecutive MFMAs share the Q fragment and feed different accumulators).  One LDS read pipeline runs
    // through all 32 MFMAs.
    // The buffer parity PAR of the phase is a compile-time constant: V^T(j) is read from buffer pair PAR, K(j+1)
    // from pair PAR ^ 1.
    auto mfma_phase = [&](auto qk_tag, auto par_tag) __attribute__((always_inline)) {
        constexpr bool WITH_QK = decltype(qk_tag)::value;
        constexpr uint32_t VP = decltype(par_tag)::value * kBufBytes;
        constexpr uint32_t KP = (decltype(par_tag)::value ^ 1) * kBufBytes;
        bf16x8 vf[16], kf[16];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) vf[u] = lds_read_b128(lds0 + va[u >> 2] + (VP + (u & 3) * 32 * 128));
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int tt = u >> 2, b = u & 3;
            uint4v p4 = {pw[4 * tt], pw[4 * tt + 1], pw[4 * tt + 2], pw[4 * tt + 3]};
            oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[u], __builtin_bit_cast(bf16x8, p4), oacc[b], 0, 0, 0);
            const int n = u + kAhead;
            if (n < 16)
                vf[n] = lds_read_b128(lds0 + va[n >> 2] + (VP + (n & 3) * 32 * 128));
            else if (WITH_QK)
                kf[n - 16] = lds_read_b128(lds0 + ka[(n - 16) >> 1] + (KP + ((n - 16) & 1) * 32 * kRowBytes));
        }
        if (WITH_QK) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                sacc[0][i] = 0.0f;
                sacc[1][i] = 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                sacc[u & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[u], qf[u >> 1], sacc[u & 1], 0, 0, 0);
                const int n = u + kAhead;
                if (n < 16) kf[n] = lds_read_b128(lds0 + ka[n >> 1] + (KP + (n & 1) * 32 * kRowBytes));
            }
        }
        SGB(DSR, kAhead);
#pragma unroll
        for (int u = 0; u < (WITH_QK ? 32 : 16) - kAhead; ++u) {
            SGB(MFMA, 1);
            SGB(DSR, 1);
        }
        SGB(MFMA, kAhead);
    };
    // S^T of tile 0 (prologue only)
    auto qk_mfmas = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            sacc[0][i] = 0.0f;
            sacc[1][i] = 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u)
            sacc[u >> 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                lds_read_b128(lds0 + ka[u & 7] + (u >> 3) * 32 * kRowBytes), qf[u & 7], sacc[u >> 3], 0, 0, 0);
    };
    // ---- ping-pong schedule.  K tile j lives in K buffer j & 1, V^T tile j in V buffer j & 1.
    // The 8 waves form two groups of 4 (one wave of each group per SIMD).  Each wave alternates a VALU
    // phase (exponentials of tile j) and an MFMA phase (second product of tile j, first product of
    // tile j+1), with a workgroup barrier after every phase.  Group 1 runs one phase behind group 0,
    // so on every SIMD one wave is in its MFMA phase while the other is in its VALU phase.  Group 1
    // also streams the tiles: during its VALU phase for tile j the buffers of V^T(j+1) and K(j+2) are
    // free (both groups are past the MFMA phase that read them), and the copies are waited for at the
    // end of its following MFMA phase, one phase before group 0 needs them.  Every wave executes the
    // same number of barriers: group 1 one more at the start, group 0 one more at the end.
    const int grp = wave >> 2, wig = wave & 3;
    using W4 = std::integral_constant<int, 4>;
    using W8 = std::integral_constant<int, 8>;
    dma_k_tile(tile_begin, 0, wave, W8{});
    dma_v_tile(tile_begin, 0, wave, W8{});
    if (tile_begin + 1 < tile_end) dma_k_tile(tile_begin + 1, 1, wave, W8{});
    // The Q fragment must be resident before the loop starts: a load still counted as pending at the
    // loop header would make the compiler wait on the vector-memory counter inside the loop.
#pragma unroll
    for (int s = 0; s < D / 16; ++s) asm volatile("" ::"v"(qf[s]));
    wait_dma();
    PHASE_BARRIER();
    if (grp == 1) PHASE_BARRIER();
    qk_mfmas();                    // S^T of the first tile (K buffer 0)
    // fast form: the first tile's row max is the offset of the whole sweep (nothing is accumulated yet, so
    // nothing needs rescaling; rows past the last key were filled with copies of it and cannot raise the max)
    if (!EXACT) m_c = tile_row_max();
    PHASE_BARRIER();

    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    // One tile that has a successor: VALU phase of tile j, then the MFMA phase (second product of tile j from
    // V buffer PAR, first product of tile j+1 from K buffer PAR ^ 1).
    auto tile_step = [&](int64_t j, auto par_tag) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_tag)::value;
        if (grp == 1) {
            dma_v_tile(j + 1, PAR ^ 1, wig, W4{});
            if (j + 2 < tile_end) dma_k_tile(j + 2, PAR, wig, W4{});
        }
        softmax_tile(j);
        PHASE_BARRIER();
        // The wave in its MFMA phase gets issue priority over its SIMD neighbour, which is in its VALU phase.
        __builtin_amdgcn_s_setprio(3);
        mfma_phase(std::true_type{}, par_tag);
        __builtin_amdgcn_s_setprio(0);
        if (grp == 1) wait_dma();
        PHASE_BARRIER();
    };
    // last tile: no next tile to prefetch or to start
    auto last_step = [&](int64_t j, auto par_tag) __attribute__((always_inline)) {
        softmax_tile(j);
        PHASE_BARRIER();
        mfma_phase(std::false_type{}, par_tag);
        PHASE_BARRIER();
    };
    // the loop is unrolled by two so that the buffer parity is a constant in each copy
    int64_t j = tile_begin;
    for (; j + 2 < tile_end; j += 2) {
        tile_step(j, P0{});
        tile_step(j + 1, P1{});
    }
    if (j + 1 < tile_end) {
        tile_step(j, P0{});
        last_step(j + 1, P1{});
    } else {
        last_step(j, P0{});
    }
    if (grp == 0) PHASE_BARRIER();

    const float l_tot = xhalf_sum(l_run);
    if (!EXACT) {
        // Did a row outgrow its offset?  Its row sum then passed 2^80, or is infinite or NaN (the comparison is
        // written so that those fail it too).  The workgroup decides as one: it stores either all of its rows or
        // none and leaves them to the exact launch.
        const bool outgrew = __builtin_amdgcn_ballot_w64(!(l_tot <= kBig)) != 0;
        if (lane == 0) wave_outgrew[wave] = outgrew ? 1u : 0u;
        __syncthreads();
        uint32_t any = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) any |= wave_outgrew[w];
        if (tid == 0) redo[blockIdx.x] = any;
        if (any) return;
    }
    if (pslot >= 0) {
        // a key-range share of an item: unnormalised accumulators, running max and row sum go to the
        // workspace; merge_partials_kernel combines the shares
        float *pp = partial + pslot * kPartialFloats;
        const int row = wave * 32 + qc;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<float4 *>(pp + row * D + 32 * b + 8 * g + 4 * hf) =
                    make_float4(oacc[b][4 * g], oacc[b][4 * g + 1], oacc[b][4 * g + 2], oacc[b][4 * g + 3]);
        if (hf == 0) {
            pp[kBq * D + row] = m_c;
            pp[kBq * D + kBq + row] = l_tot;
        }
        return;
    }
    const float inv = 1.0f / l_tot;
    const int64_t rr = r0 + qc;
    if (rr >= k_sel) return;
    // compact output row rr, or straight into the cached buffer's row of that token
    const int64_t orow = o_scatter ? (int64_t)idx_sel[rr] : rr;
    __bf16 *op = o_sel + orow * o_stride_n + (int64_t)head * D;
    if (!o_scatter || (uint64_t)orow < (uint64_t)N)     // a row index outside the cached buffer writes nothing
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            // registers 4g..4g+3: head-dim 32*b + 8*g + 4*hf + 0..3
            uint2v o4;
            o4[0] = pack_bf16(oacc[b][4 * g] * inv, oacc[b][4 * g + 1] * inv);
            o4[1] = pack_bf16(oacc[b][4 * g + 2] * inv, oacc[b][4 * g + 3] * inv);
            *reinterpret_cast<uint2v *>(op + 32 * b + 8 * g + 4 * hf) = o4;
        }
    if (lse_sel && hf == 0) lse_sel[rr * H + head] = (m_c + log2f(l_tot)) * 0.69314718055994530942f;
}


// Combines the key-range shares of the split items: with m* = max_s m_s and w_s = 2^(m_s - m*),
// O = sum_s w_s O_s / sum_s w_s l_s.  Workgroup (x, y) handles rows 8*y .. 8*y+7 of split item x; a
// thread handles one row and four head-dim elements.
__global__ __launch_bounds__(256) void merge_partials_kernel(const float *__restrict__ partial, AttnSchedule sch,
                                                             int32_t H, int64_t k_sel, int64_t n_rows,
                                                             const int32_t *__restrict__ idx_sel, __bf16 *__restrict__ o_sel,
                                                             int64_t o_stride_n, int o_scatter,
                                                             float *__restrict__ lse_sel)
{
    const int64_t left = sch.items_per_xcd - sch.full_items;
    const int64_t xcd = blockIdx.x / left, li = blockIdx.x % left;
    const int64_t item = xcd * sch.items_per_xcd + sch.full_items + li;
    if (item >= (xcd + 1) * sch.items_per_xcd || item >= (int64_t)H * sch.q_tiles) return;
    const int head = (int)(item / sch.q_tiles);
    const int64_t qt = item % sch.q_tiles;
    const float *base = partial + (xcd * left + li) * sch.splits * (int64_t)kPartialFloats;
    const int d4 = (threadIdx.x & 31) * 4;
    {
        const int row = (threadIdx.x >> 5) + 8 * blockIdx.y;
        const int64_t rr = qt * kBq + row;
        if (rr >= k_sel) return;
        float m_star = -INFINITY;
        for (int s = 0; s < sch.splits; ++s) m_star = fmaxf(m_star, base[s * (int64_t)kPartialFloats + kBq * D + row]);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float l = 0.0f;
        for (int s = 0; s < sch.splits; ++s) {
            const float *ps = base + s * (int64_t)kPartialFloats;
            const float w = exp2f(ps[kBq * D + row] - m_star);
            const float4 o = *reinterpret_cast<const float4 *>(ps + row * D + d4);
            acc.x += w * o.x;
            acc.y += w * o.y;
            acc.z += w * o.z;
            acc.w += w * o.w;
            l += w * ps[kBq * D + kBq + row];
        }
        const float inv = 1.0f / l;
        uint2v o4;
        o4[0] = pack_bf16(acc.x * inv, acc.y * inv);
        o4[1] = pack_bf16(acc.z * inv, acc.w * inv);
        const int64_t orow = o_scatter ? (int64_t)idx_sel[rr] : rr;
        if (!o_scatter || (uint64_t)orow < (uint64_t)n_rows)
            *reinterpret_cast<uint2v *>(o_sel + orow * o_stride_n + (int64_t)head * D + d4) = o4;
        if (lse_sel && d4 == 0) lse_sel[rr * H + head] = (m_star + log2f(l)) * 0.69314718055994530942f;
    }
}

}  // namespace

// The budget-aware split for k_sel selected queries of H heads over N keys; `slots` = workgroups per XCD.
// False when the grid would not fit.
static bool plan_attn(int64_t N, int32_t H, int64_t k_sel, AttnSchedule &sch, int64_t &slots)
{
    const int64_t ntiles = (N + kBk - 1) / kBk;
    constexpr int kCuPerXcd = 32;
    sch.q_tiles = (int32_t)((k_sel + kBq - 1) / kBq);
    const int64_t total = (int64_t)sch.q_tiles * H;
    sch.items_per_xcd = (total + kNumXcd - 1) / kNumXcd;
    // Items that would run in a last, partly filled round are cut along the keys into `splits` shares
    // each, chosen (up to 8 shares per item, 64 shares per XCD) so that the shares take the fewest
    // rounds relative to their length: rounds(left * splits) / splits is the tail's cost in full sweeps.
    int64_t left = sch.items_per_xcd % kCuPerXcd;
    int64_t splits = 1;
    if (left > 0) {
        double best = 1.0;
        for (int64_t s2 = 2; s2 <= 8 && left * s2 <= kMaxSharesPerXcd && s2 <= ntiles; ++s2) {
            if ((s2 - 1) * ((ntiles + s2 - 1) / s2) >= ntiles) continue;      // would leave an empty share
            const double cost = (double)((left * s2 + kCuPerXcd - 1) / kCuPerXcd) / (double)s2;
            if (cost < best - 1e-9) {
                best = cost;
                splits = s2;
            }
        }
    }
    if (splits <= 1) {
        left = 0;
        splits = 1;
    }
    sch.full_items = sch.items_per_xcd - left;
    sch.splits = (int32_t)splits;
    sch.tiles_per_split = (ntiles + splits - 1) / splits;
    slots = sch.full_items + left * splits;
    return slots * kNumXcd <= 2147483647LL && ntiles <= 2147483647LL;
}

int attn_bf16_plan(int64_t N, int32_t H, int64_t k_sel, int64_t plan[8])
{
    AttnSchedule sch;
    int64_t slots = 0;
    if (!plan_attn(N, H, k_sel, sch, slots)) return fail(ASTRAEA_ERR_INVALID, "astraea_attn_plan: grid too large");
    plan[0] = sch.q_tiles;
    plan[1] = sch.items_per_xcd;
    plan[2] = sch.full_items;
    plan[3] = sch.splits;
    plan[4] = sch.tiles_per_split;
    plan[5] = slots * kNumXcd;
    plan[6] = (N + kBk - 1) / kBk;
    plan[7] = (int64_t)kNumXcd * kMaxSharesPerXcd;
    return ASTRAEA_OK;
}

// Workspace of the bf16 path: the V^T tiles written by the pre-pass, then the partial results of the
// split items (at most kMaxSharesPerXcd shares per XCD), then one redo flag per workgroup of the largest
// grid a selection of up to N queries can launch.
static size_t vt_bytes(int64_t N, int32_t H)
{
    const int64_t ntiles = (N + kBk - 1) / kBk;
    return (size_t)ntiles * (size_t)H * kTileBytes;
}
static size_t partial_bytes() { return (size_t)kNumXcd * kMaxSharesPerXcd * kPartialFloats * sizeof(float); }
// Workgroups of a launch: 8 * (full items + shares) per XCD <= all items rounded up to the XCD count, plus the shares.
static size_t redo_flags(int64_t N, int32_t H)
{
    const int64_t items = ((N + kBq - 1) / kBq) * (int64_t)H;
    return (size_t)(((items + kNumXcd - 1) / kNumXcd) * kNumXcd + (int64_t)kNumXcd * kMaxSharesPerXcd);
}
size_t attn_bf16_workspace_bytes(int64_t N, int32_t H)
{
    if (N <= 0 || H <= 0) return 0;
    const size_t b = vt_bytes(N, H) + partial_bytes() + redo_flags(N, H) * sizeof(uint32_t);
    return (b + 255) & ~(size_t)255;
}

int launch_attn_bf16_d128(const void *q, const void *k, const void *v, int64_t N, int32_t H, int64_t q_stride_n,
                          int64_t q_stride_h, int64_t kv_stride_n, int64_t kv_stride_h, const int32_t *idx_sel,
                          int64_t k_sel, int q_is_compact, float scale, void *o_sel, int64_t o_stride_n, int o_scatter,
                          float *lse_sel, void *workspace,
                          hipStream_t stream)
{
    if (k_sel == 0) return ASTRAEA_OK;
    // a tile's lane offsets are 32-bit: 64 rows must span less than 4 GiB
    if (kv_stride_n * 2 * kBk >= (int64_t)1 << 32)
        return fail(ASTRAEA_ERR_UNSUPPORTED, "astraea_sparse_attn_fwd: K/V token stride too large");
    const int64_t ntiles = (N + kBk - 1) / kBk;
    AttnSchedule sch;
    int64_t slots = 0;
    if (!plan_attn(N, H, k_sel, sch, slots))
        return fail(ASTRAEA_ERR_INVALID, "astraea_sparse_attn_fwd: grid too large");
    const int64_t left = sch.items_per_xcd - sch.full_items;
    char *vt = (char *)workspace;
    float *partial = (float *)(vt + vt_bytes(N, H));
    uint32_t *redo = (uint32_t *)((char *)partial + partial_bytes());
    // compact queries may outnumber the keys (cross-attention of many rows over a short context): the flag
    // area is sized for up to N queries, larger selections run the exact form alone, which needs no flags
    const bool two_forms = (size_t)(slots * kNumXcd) <= redo_flags(N, H);
    hipLaunchKernelGGL(transpose_v_kernel, dim3((unsigned)ntiles, (unsigned)H), dim3(256), 0, stream,
                       (const __bf16 *)v, N, kv_stride_n, kv_stride_h, ntiles, vt);
    dim3 grid((unsigned)(slots * kNumXcd)), block(kWaves * kWave);
    const float c = scale * 1.44269504088896340736f;
    kernel_timer_begin(stream);
    if (two_forms)
        hipLaunchKernelGGL(attn_bf16_kernel<false>, grid, block, 0, stream, (const __bf16 *)q, (const __bf16 *)k,
                           (const char *)vt, N, H, q_stride_n, q_stride_h, kv_stride_n, kv_stride_h, idx_sel, k_sel,
                           q_is_compact, c, (__bf16 *)o_sel, o_stride_n, o_scatter, lse_sel, sch, partial, redo);
    else
        hipLaunchKernelGGL(attn_bf16_kernel<true>, grid, block, 0, stream, (const __bf16 *)q, (const __bf16 *)k,
                           (const char *)vt, N, H, q_stride_n, q_stride_h, kv_stride_n, kv_stride_h, idx_sel, k_sel,
                           q_is_compact, c, (__bf16 *)o_sel, o_stride_n, o_scatter, lse_sel, sch, partial,
                           (uint32_t *)nullptr);
    kernel_timer_end(stream);
    // the exact form over the same grid: only workgroups that flagged themselves do anything
    if (two_forms)
        hipLaunchKernelGGL(attn_bf16_kernel<true>, grid, block, 0, stream, (const __bf16 *)q, (const __bf16 *)k,
                           (const char *)vt, N, H, q_stride_n, q_stride_h, kv_stride_n, kv_stride_h, idx_sel, k_sel,
                           q_is_compact, c, (__bf16 *)o_sel, o_stride_n, o_scatter, lse_sel, sch, partial, redo);
    if (left > 0)
        hipLaunchKernelGGL(merge_partials_kernel, dim3((unsigned)(left * kNumXcd), kBq / 8), dim3(256), 0, stream, partial, sch,
                           H, k_sel, N, idx_sel, (__bf16 *)o_sel, o_stride_n, o_scatter, lse_sel);
    return check_launch("astraea_sparse_attn_fwd(bf16)");
}

}  // namespace astraea
