// bf16 GEMM  out = epilogue(A W^T + bias)  for gfx950, fp32 accumulation on the matrix cores.
//
// This is the "24 b L_q C^2" term of the per-layer cost in Appendix B of the paper (QKV, output
// and FFN projections), plus the cross-attention projections the cost model leaves out.
//
// Design
//   * Both operands are K-contiguous (activations [M, K], weights [N, K]), so the A and B fragments
//     of v_mfma_f32_32x32x16_bf16 are plain 16-byte loads: lane l holds row (l % 32) and the eight
//     k values 8 * (l / 32) .. +7 of a 16-wide k step.
//   * A workgroup is 4 waves stacked along M.  Wave tile = (32 TM) x (32 TN); workgroup tile =
//     (128 TM) x (32 TN) x 64.  TN runs from 2 to 8 so that the tile count can be matched to the
//     256 compute units for the skinny M = 1024 shapes of the streaming chunk.
//   * Tiles go global -> registers -> LDS (two LDS stages, two or three register sets: a load is in
//     flight for two or three k iterations), one barrier per k tile.  LDS rows are 64 bf16 (128 B); the
//     16-byte chunk index is XOR-ed with (row / 2) % 8 so that fragment reads are conflict free on the
//     64-bank LDS.
//   * Workgroup ids are spread round-robin over the 8 XCDs by the hardware; the kernel undoes that
//     so that each XCD (one L2) owns a contiguous range of tiles, ordered in groups of M tiles that
//     share weight tiles.
//   * Split-K, for the one kind of shape that needs it (few output tiles, long k: FFN-2 of the small model),
//     is two launches: the parts store fp32 partial sums, an elementwise kernel adds them in k order and applies
//     the epilogue.  fp32 atomics on the output cost ~40 us per 1.5 M elements here, and a last-arriver
//     reduction inside one launch needs device-scope fences that write back and invalidate the whole L2 of an
//     XCD (measured +100 us on a 64 us launch).
#include "common.h"

#include <mutex>
#include <type_traits>

#include <stdio.h>
#include <stdlib.h>

namespace sdv2 {

namespace {

// Epilogue.  Accumulator register r of a 32x32 block holds row 8 (r / 4) + 4 (lane / 32) + r % 4 and
// column lane % 32, which is a poor shape for memory (2-byte or 4-byte pieces of many rows).  Each wave
// therefore passes its accumulators through a private LDS region, 32 rows x 64 columns at a time, and
// reads them back row-major so that a lane owns four consecutive columns: stores become 8-byte (bf16)
// or 16-byte (fp32) pieces that fill whole 128- or 256-byte row segments, and the read-modify-write
// epilogues issue all their loads of x before the first use.
constexpr int EPI_LD = 68;                          // floats per LDS row: 64 + 4 of padding
constexpr int EPI_WAVE_FLOATS = 32 * EPI_LD;

template <int EPI, int NB>
__device__ __forceinline__ void epilogue_chunk(const GemmArgs& g, const f32x16& acc0, const f32x16& acc1, float* stage,
                                               int row_base, int col_base, int lane) {
    const int l31 = lane & 31, lh = lane >> 5;
    __builtin_amdgcn_sched_barrier(0);               // one chunk at a time: bounds the registers in flight
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + 4 * lh + (r & 3);
        stage[row * EPI_LD + l31] = acc0[r];
        if (NB == 2) stage[row * EPI_LD + 32 + l31] = acc1[r];
    }
    constexpr int kLanesPerRow = NB * 8;
    constexpr int kRowsPerPass = 64 / kLanesPerRow;
    constexpr int kPasses = 32 / kRowsPerPass;
    const int prow = lane / kLanesPerRow;
    const int c4 = (lane % kLanesPerRow) * 4;
    const int gcol = col_base + c4;
    const bool col_ok = gcol < g.N;                  // N is a multiple of 4: all four columns or none
    const int gcolc = col_ok ? gcol : 0;
    f32x4 bias = {0.0f, 0.0f, 0.0f, 0.0f};
    if (g.bias != nullptr) bias = *reinterpret_cast<const f32x4*>(g.bias + gcolc);
    f32x4 gate_a = {0.0f, 0.0f, 0.0f, 0.0f};
    if (EPI == kEpiGatedResidual) gate_a = *reinterpret_cast<const f32x4*>(g.gate_a + gcolc);
    // passes are handled four at a time: all loads of x and of the gate first, then the arithmetic and stores
    constexpr int kGroup = kPasses < 4 ? kPasses : 4;
#pragma unroll
    for (int p0 = 0; p0 < kPasses; p0 += kGroup) {
        f32x4 xv[kGroup];
        f32x4 gb[kGroup];
        if (EPI == kEpiGatedResidual || EPI == kEpiResidual) {
#pragma unroll
            for (int q = 0; q < kGroup; ++q) {
                const int grow = row_base + (p0 + q) * kRowsPerPass + prow;
                const bool ok = col_ok && grow < g.M;
                const int growc = ok ? grow : 0;
                xv[q] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(g.out) + (size_t)growc * g.N + gcolc);
                if (EPI == kEpiGatedResidual)
                    gb[q] = *reinterpret_cast<const f32x4*>(g.gate_b + (size_t)(growc / g.rows_per_gate) * g.gate_b_stride + gcolc);
            }
        }
#pragma unroll
        for (int q = 0; q < kGroup; ++q) {
            const int row = (p0 + q) * kRowsPerPass + prow;
            const int grow = row_base + row;
            f32x4 v = *reinterpret_cast<const f32x4*>(stage + row * EPI_LD + c4);
            v += bias;
            if (col_ok && grow < g.M) {
                const size_t o = (size_t)grow * g.N + gcol;
                if (EPI == kEpiPartial) {
                    *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.out) + o) = v;
                } else if (EPI == kEpiBias || EPI == kEpiBiasGelu) {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (bf16)(EPI == kEpiBiasGelu ? gelu_tanh_f(v[e]) : v[e]);
                    *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16*>(g.out) + o) = w;
                } else {
                    if (EPI == kEpiGatedResidual) v *= (gate_a + gb[q]);
                    *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.out) + o) = xv[q] + v;
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// row0: first output row of this wave's tile; col0: first output column of the workgroup's tile.
template <int TM, int TN, int EPI>
__device__ __forceinline__ void epilogue(const GemmArgs& g, f32x16 (&acc)[TM][TN], float* stage, int row0, int col0,
                                         int lane) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int jc = 0; jc < (TN + 1) / 2; ++jc) {
            if (2 * jc + 1 < TN)
                epilogue_chunk<EPI, 2>(g, acc[i][2 * jc], acc[i][2 * jc + 1], stage, row0 + 32 * i, col0 + 64 * jc, lane);
            else
                epilogue_chunk<EPI, 1>(g, acc[i][2 * jc], acc[i][2 * jc], stage, row0 + 32 * i, col0 + 64 * jc, lane);
        }
    }
}

template <int TM, int TN>
__device__ __forceinline__ void run_epilogue(const GemmArgs& g, f32x16 (&acc)[TM][TN], float* stage, int row0, int col0,
                                             int lane) {
    switch (g.epilogue) {
        case kEpiBias: epilogue<TM, TN, kEpiBias>(g, acc, stage, row0, col0, lane); break;
        case kEpiBiasGelu: epilogue<TM, TN, kEpiBiasGelu>(g, acc, stage, row0, col0, lane); break;
        case kEpiGatedResidual: epilogue<TM, TN, kEpiGatedResidual>(g, acc, stage, row0, col0, lane); break;
        case kEpiPartial: epilogue<TM, TN, kEpiPartial>(g, acc, stage, row0, col0, lane); break;
        default: epilogue<TM, TN, kEpiResidual>(g, acc, stage, row0, col0, lane); break;
    }
}

// Tiles whose k loop fits in 256 registers are compiled for two workgroups per compute unit, so that one
// workgroup's barrier and LDS-latency bubbles are filled by the other's MFMAs.  BK (64 or 128) is the k
// depth of an LDS stage: a deeper stage halves the number of barriers, which is what the small tiles
// (few MFMAs per barrier) are short of.
// PF is the number of register sets = how many k tiles ahead the global loads run.  A compute unit needs
// on the order of 100 KB of loads in flight to cover the L2 latency; tiles that run one workgroup per
// unit get there with three sets, small tiles with two sets and two or three workgroups per unit.
template <int TM, int TN, int BK, int PF>
__global__ __launch_bounds__(256, ((TM * TN <= 5 && BK == 64 && PF == 2) ? 2 : 1)) void gemm_kernel(GemmArgs g, int tiles_m,
                                                                                                  int tiles_n, int group_m,
                                                                                                  int splitk) {
    constexpr int BM = 128 * TM;
    constexpr int BN = 32 * TN;
    constexpr int CPR = BK / 8;                 // 16-byte chunks per LDS row
    constexpr int RPP = 256 / CPR;              // tile rows covered by one pass of the 256 threads
    constexpr int NA = BM / RPP;                // 16-byte chunks of the A tile per thread
    constexpr int NB = BN / RPP;                // of the W tile
    constexpr int KS = BK / 16;                 // MFMA k steps per stage
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* const sm = reinterpret_cast<bf16*>(smem_raw);     // [2][BM*BK | BN*BK]
    constexpr int STAGE = (BM + BN) * BK;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l31 = lane & 31;
    const int lh = lane >> 5;

    // ---- which tile: undo the round-robin XCD dispatch, then grouped ordering
    const int nwg = gridDim.x;                                   // multiple of 8
    const int logical = (blockIdx.x & 7) * (nwg >> 3) + (blockIdx.x >> 3);
    const int tiles = tiles_m * tiles_n;
    if (logical >= tiles * splitk) return;
    const int ks = logical / tiles;                              // which part of k (0 when k is not split)
    const int t = logical - ks * tiles;
    const int group_size = group_m * tiles_n;
    const int grp = t / group_size;
    const int first_m = grp * group_m;
    const int gm = min(tiles_m - first_m, group_m);
    const int in_grp = t - grp * group_size;
    const int tile_m = first_m + in_grp % gm;
    const int tile_n = in_grp / gm;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;

    const int KT = g.K / BK;
    const int kt0 = (int)((long long)ks * KT / splitk);
    const int kt1 = (int)((long long)(ks + 1) * KT / splitk);
    if (splitk > 1) {                                            // this part's fp32 partial sums, plain stores
        g.out = g.splitk_partials + (size_t)ks * g.M * g.N;
        g.epilogue = kEpiPartial;
        g.bias = nullptr;
    }

    // ---- global -> register staging
    const int crow = tid / CPR;
    const int cchunk = tid % CPR;
    const bf16* ap[NA];
    const bf16* bp[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int row = min(m0 + crow + RPP * i, g.M - 1);
        ap[i] = g.a + (size_t)row * g.K + cchunk * 8;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int row = min(n0 + crow + RPP * i, g.N - 1);
        bp[i] = g.w + (size_t)row * g.K + cchunk * 8;
    }
    // LDS swizzle: the 16-byte chunk c of row r is stored at position c ^ ((r / 2) % 8).  The LDS has 64
    // banks (256 bytes per clock); a row is 128 bytes, so rows r and r + 1 fall in different bank halves
    // and the sixteen lanes that a b128 read serves per clock (rows r .. r + 15, same chunk) then hit
    // sixteen different 16-byte slots.  (XOR with r % 8, the 32-bank recipe, reads at half rate here.)
    // RPP is a multiple of 16, so ((row / 2) % 8) of every chunk this thread stages is that of crow.
    const int st_off = crow * BK + ((cchunk ^ ((crow >> 1) & 7)) << 3);
    // PF register sets: tile t lives in set t % PF from its load until it is written to LDS stage t % 2
    // at the end of iteration t - 1, so a global load has PF iterations of MFMA work to hide behind.
    bf16x8 ra[PF][NA], rb[PF][NB];

    auto gload = [&](bf16x8 (&xa)[NA], bf16x8 (&xb)[NB], int kt) {
#pragma unroll
        for (int i = 0; i < NA; ++i) xa[i] = *reinterpret_cast<const bf16x8*>(ap[i] + kt * BK);
#pragma unroll
        for (int i = 0; i < NB; ++i) xb[i] = *reinterpret_cast<const bf16x8*>(bp[i] + kt * BK);
    };
    auto sstore = [&](const bf16x8 (&xa)[NA], const bf16x8 (&xb)[NB], int buf) {
        bf16* sa = sm + buf * STAGE;
        bf16* sb = sa + BM * BK;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<bf16x8*>(sa + st_off + i * RPP * BK) = xa[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *reinterpret_cast<bf16x8*>(sb + st_off + i * RPP * BK) = xb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int a_row0 = wave * (32 * TM) + l31;
    // One stage = KS 16-wide steps.  The fragments of step s + 1 are read from LDS before the MFMAs of
    // step s are issued, so that the LDS latency hides behind matrix work.
    auto load_frags = [&](bf16x8 (&fa)[TM], bf16x8 (&fb)[TN], const bf16* sa, const bf16* sb, int s) {
        const int coff = ((2 * s + lh) ^ ((l31 >> 1) & 7)) << 3;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = *reinterpret_cast<const bf16x8*>(sa + (a_row0 + 32 * i) * BK + coff);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[j] = *reinterpret_cast<const bf16x8*>(sb + (l31 + 32 * j) * BK + coff);
    };
    auto compute = [&](int buf) {
        const bf16* sa = sm + buf * STAGE;
        const bf16* sb = sa + BM * BK;
        bf16x8 fa[2][TM], fb[2][TN];
        load_frags(fa[0], fb[0], sa, sb, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (s + 1 < KS) load_frags(fa[(s + 1) & 1], fb[(s + 1) & 1], sa, sb, s + 1);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s & 1][i], fb[s & 1][j], acc[i][j], 0, 0, 0);
        }
    };

    // Issue order of one half iteration.  A wave issues in order, and a global load or an LDS write
    // occupies its issue slot for tens of cycles; so they are spread between the MFMAs (whose 32-cycle
    // execution leaves issue slots free) instead of being issued in a burst before or after them:
    //   first step's fragment reads | per MFMA: 1 MFMA, fragment reads of the next step, then one
    //   global load (tile i + 2) in the first half of the MFMAs and one LDS write (tile i + 1) in the
    //   second half.
    auto issue_pipeline = [&]() {
        constexpr int kMfma = TM * TN * KS;
        constexpr int kReadsPerMfma = (TM + TN + TM * TN - 1) / (TM * TN);
        constexpr int kMem = NA + NB;
        constexpr int kMemPerMfma = (2 * kMem + kMfma - 1) / kMfma;
        __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
#pragma unroll
        for (int m = 0; m < kMfma; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, kReadsPerMfma, 0);
            if (m < kMfma / 2) __builtin_amdgcn_sched_group_barrier(0x020, kMemPerMfma, 0);
            else __builtin_amdgcn_sched_group_barrier(0x200, kMemPerMfma, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // Loads are unconditional (the tile index is clamped, the tail re-reads the last tile) so that a step
    // has no control flow around them and they stay in flight across the MFMA work.  Step k of the
    // unrolled body: tile t sits in LDS stage k % 2; load tile t + PF into set k % PF (free since tile t
    // was written out), compute, write set (k + 1) % PF (tile t + 1) to the other stage.
    const int nk = kt1 - kt0;
    const int kt_last = kt1 - 1;
    auto step = [&](auto kc, int t) {
        constexpr int k = decltype(kc)::value;
        __builtin_amdgcn_sched_barrier(0);
        gload(ra[k % PF], rb[k % PF], min(kt0 + t + PF, kt_last));
        compute(k % 2);
        sstore(ra[(k + 1) % PF], rb[(k + 1) % PF], (k + 1) % 2);
        issue_pipeline();
        __syncthreads();
    };
    if (nk > 0) {
#pragma unroll
        for (int p = 0; p < PF; ++p) gload(ra[p], rb[p], min(kt0 + p, kt_last));
        sstore(ra[0], rb[0], 0);
    }
    __syncthreads();
    constexpr int U = (PF % 2 == 0) ? PF : 2 * PF;      // unroll so that stage and set indices are constants
    int i = 0;
    for (; i + U <= nk; i += U) {
        step(std::integral_constant<int, 0>{}, i);
        step(std::integral_constant<int, 1>{}, i + 1);
        if constexpr (U > 2) {
            step(std::integral_constant<int, 2>{}, i + 2);
            step(std::integral_constant<int, 3>{}, i + 3);
            step(std::integral_constant<int, 4>{}, i + 4);
            step(std::integral_constant<int, 5>{}, i + 5);
        }
    }
    // tail: fewer than U tiles left; the last tile needs no write-out but doing one is harmless
    if (i < nk) step(std::integral_constant<int, 0>{}, i);
    if constexpr (U > 2) {
        if (i + 1 < nk) step(std::integral_constant<int, 1>{}, i + 1);
        if (i + 2 < nk) step(std::integral_constant<int, 2>{}, i + 2);
        if (i + 3 < nk) step(std::integral_constant<int, 3>{}, i + 3);
        if (i + 4 < nk) step(std::integral_constant<int, 4>{}, i + 4);
    }

    // ---- epilogue (the LDS stages are free once every wave has left the k loop)
    __syncthreads();
    float* stage = reinterpret_cast<float*>(smem_raw) + wave * EPI_WAVE_FLOATS;
    run_epilogue<TM, TN>(g, acc, stage, m0 + wave * (32 * TM), n0, lane);
}

// ---------------------------------------------------------------------------------------------------
// Second kernel: tiles go global -> LDS directly (global_load_lds_dwordx4, no staging registers and no
// LDS write instructions), 8 waves per workgroup arranged WM x WN so that a wave's tile is (32 TM) x (32 TN)
// with TM + TN fragment reads per TM TN MFMAs, NS LDS stages of BK = 64.
//
// A direct load writes 16 bytes per lane at consecutive LDS addresses (lane l -> base + 16 l), so one wave
// instruction fills 8 tile rows of 128 bytes.  The swizzle is applied on the global side: the lane that
// fills chunk position p of row r fetches logical chunk p ^ ((r / 2) % 8) of that row; the 8 lanes of a row
// still cover one whole 128-byte segment of the operand.
//
// Iteration t:  wait for this wave's loads of tile t | barrier (tile t visible to all; every wave is done
// with tile t - 1, whose stage is therefore free) | issue the loads of tile t + NS - 1 | compute tile t.
constexpr int kVmcntShift = 14;
constexpr int vmcnt_imm(int n) {      // s_waitcnt with only vmcnt constrained
    return (n & 0xF) | ((n >> 4) << kVmcntShift) | 0x0F70;
}
typedef __attribute__((address_space(3))) void* lds_void_ptr;
// 16 bytes per lane from global memory straight into LDS at dst + 16 * lane (dst is wave-uniform).
__device__ __forceinline__ void load_to_lds_b128(const void* src, void* dst) {
    __builtin_amdgcn_global_load_lds(src, (lds_void_ptr)dst, 16, 0, 0);
}

template <int WM, int WN, int TM, int TN, int NS>
__global__ __launch_bounds__(64 * WM * WN, 1) void gemm_dma_kernel(GemmArgs g, int tiles_m, int tiles_n,
                                                                   int group_m, int splitk) {
    constexpr int NW = WM * WN;
    constexpr int BK = 64;
    constexpr int BM = 32 * TM * WM;
    constexpr int BN = 32 * TN * WN;
    constexpr int KS = BK / 16;
    constexpr int GROUPS = (BM + BN) / 8;            // 8-row groups of the stacked [A; W] tile = wave loads per tile
    constexpr int LPW = GROUPS / NW;                 // loads per wave per tile
    static_assert(GROUPS % NW == 0, "tile rows must split evenly over the waves");
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN;
    const int wn = wave % WN;
    const int l31 = lane & 31;
    const int lh = lane >> 5;

    const int nwg = gridDim.x;                                   // multiple of 8
    const int logical = (blockIdx.x & 7) * (nwg >> 3) + (blockIdx.x >> 3);
    const int tiles = tiles_m * tiles_n;
    if (logical >= tiles * splitk) return;
    const int ks = logical / tiles;                              // which part of k (0 when k is not split)
    const int t = logical - ks * tiles;
    const int group_size = group_m * tiles_n;
    const int grp = t / group_size;
    const int first_m = grp * group_m;
    const int gm = min(tiles_m - first_m, group_m);
    const int in_grp = t - grp * group_size;
    const int tile_m = first_m + in_grp % gm;
    const int tile_n = in_grp / gm;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;

    const int KT = g.K / BK;
    const int kt0 = (int)((long long)ks * KT / splitk);
    const int kt1 = (int)((long long)(ks + 1) * KT / splitk);
    const int nk = kt1 - kt0;
    if (splitk > 1) {                                            // this part's fp32 partial sums, plain stores
        g.out = g.splitk_partials + (size_t)ks * g.M * g.N;
        g.epilogue = kEpiPartial;
        g.bias = nullptr;
    }

    // ---- per-lane source of each of this wave's loads (8-row group wave + NW i of the stacked tile): a 32-bit
    // byte offset into the operand (operands are below 4 GB); the k advance is uniform
    uint32_t off[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int r = 8 * (wave + NW * i) + (lane >> 3);         // row of the stacked tile
        const int c = (lane & 7) ^ ((r >> 1) & 7);               // logical 16-byte chunk this lane fetches
        const int row = (8 * (wave + NW * i) < BM) ? min(m0 + r, g.M - 1) : min(n0 + r - BM, g.N - 1);
        off[i] = (uint32_t)row * (uint32_t)g.K * 2u + (uint32_t)c * 16u;
    }
    const unsigned char* a_base = reinterpret_cast<const unsigned char*>(g.a) + (size_t)kt0 * (BK * 2);
    const unsigned char* w_base = reinterpret_cast<const unsigned char*>(g.w) + (size_t)kt0 * (BK * 2);
    auto issue_loads = [&](int kt_rel, int stage) {
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            unsigned char* dst = smem_raw + stage * STAGE_BYTES + (wave + NW * i) * 1024;
            const unsigned char* base = (8 * (wave + NW * i) < BM) ? a_base : w_base;   // uniform per load
            load_to_lds_b128(base + (size_t)kt_rel * (BK * 2) + off[i], dst);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int a_row0 = wm * (32 * TM) + l31;
    const int b_row0 = BM + wn * (32 * TN) + l31;
    auto load_frags = [&](bf16x8 (&fa)[TM], bf16x8 (&fb)[TN], const bf16* st, int s) {
        const int coff = ((2 * s + lh) ^ ((l31 >> 1) & 7)) << 3;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(st + (a_row0 + 32 * i) * BK + coff);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(st + (b_row0 + 32 * j) * BK + coff);
    };
    auto compute = [&](int stage) {
        const bf16* st = reinterpret_cast<const bf16*>(smem_raw + stage * STAGE_BYTES);
        bf16x8 fa[2][TM], fb[2][TN];
        load_frags(fa[0], fb[0], st, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (s + 1 < KS) load_frags(fa[(s + 1) & 1], fb[(s + 1) & 1], st, s + 1);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s & 1][i], fb[s & 1][j], acc[i][j], 0, 0, 0);
        }
    };
    // Issue order of one iteration: the first step's fragment reads, then per MFMA one MFMA, the next step's
    // fragment reads spread evenly, and the tile loads spread over the first MFMAs.
    auto issue_pipeline = [&](bool with_loads) {
        constexpr int kMfma = TM * TN * KS;
        constexpr int kReadsPerMfma = (TM + TN + TM * TN - 1) / (TM * TN);
        __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
#pragma unroll
        for (int m = 0; m < kMfma; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, kReadsPerMfma, 0);
            if (with_loads && m < LPW) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    auto step = [&](auto sc, int tt) {
        constexpr int s = decltype(sc)::value;                   // stage of tile tt
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 2) * LPW));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        // Loads are unconditional (past the end they re-read the last tile into a stage nobody reads again)
        // so that the wait count above is the same in every iteration.
        issue_loads(min(tt + NS - 1, nk - 1), (s + NS - 1) % NS);
        compute(s);
        issue_pipeline(true);
    };
    if (nk > 0) {
#pragma unroll
        for (int p = 0; p < NS - 1; ++p) issue_loads(min(p, nk - 1), p);
    }
    int i = 0;
    for (; i + NS <= nk; i += NS) {
        step(std::integral_constant<int, 0>{}, i);
        if constexpr (NS > 1) step(std::integral_constant<int, 1 % NS>{}, i + 1);
        if constexpr (NS > 2) step(std::integral_constant<int, 2 % NS>{}, i + 2);
        if constexpr (NS > 3) step(std::integral_constant<int, 3 % NS>{}, i + 3);
    }
    if (i < nk) step(std::integral_constant<int, 0>{}, i);
    if constexpr (NS > 2) {
        if (i + 1 < nk) step(std::integral_constant<int, 1 % NS>{}, i + 1);
    }
    if constexpr (NS > 3) {
        if (i + 2 < nk) step(std::integral_constant<int, 2 % NS>{}, i + 2);
    }

    // ---- epilogue: every direct load has landed and every wave has left the k loop before the stages
    // are reused as staging space
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    float* stage = reinterpret_cast<float*>(smem_raw) + wave * EPI_WAVE_FLOATS;
    run_epilogue<TM, TN>(g, acc, stage, m0 + wm * (32 * TM), n0 + wn * (32 * TN), lane);
}


// ---------------------------------------------------------------------------------------------------
// Ring variant of the direct-load kernel: k tiles of 32 in a ring of four LDS stages, eight waves, a branch-free
// loop body in which a wave issues one direct load every fourth MFMA (the compute unit's loads arrive as an
// even stream three tiles ahead instead of a burst after the barrier that blocks the issuing waves) and reads
// the next k step's fragments between the MFMAs of the current one.
template <int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(512, 1) void gemm_ring_kernel(GemmArgs g, int tiles_m, int tiles_n, int group_m,
                                                           int splitk) {
    static_assert(WM * WN == 8, "eight waves");
    constexpr int NW = 8, BK = 32, NS = 4;
    constexpr int BM = 32 * TM * WM;
    constexpr int BN = 32 * TN * WN;
    constexpr int LPW = (BM + BN) / 16 / NW;         // a wave load fills 16 rows of 64 bytes
    static_assert(LPW == 4 && BM % 128 == 0, "256 x 256 tiles");
    constexpr int LPW_A = BM / 128;
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN;
    const int wn = wave % WN;
    const int l31 = lane & 31;
    const int lh = lane >> 5;

    const int nwg = gridDim.x;
    const int logical = (blockIdx.x & 7) * (nwg >> 3) + (blockIdx.x >> 3);
    const int tiles = tiles_m * tiles_n;
    if (logical >= tiles * splitk) return;
    const int ks = logical / tiles;                              // which part of k (0 when k is not split)
    const int t = logical - ks * tiles;
    const int group_size = group_m * tiles_n;
    const int grp = t / group_size;
    const int first_m = grp * group_m;
    const int gm = min(tiles_m - first_m, group_m);
    const int in_grp = t - grp * group_size;
    const int tile_m = first_m + in_grp % gm;
    const int tile_n = in_grp / gm;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;
    const int nk_all = g.K / BK;
    const int kt0 = (int)((long long)ks * nk_all / splitk);
    const int nk = (int)((long long)(ks + 1) * nk_all / splitk) - kt0;
    if (splitk > 1) {                                            // this part's fp32 partial sums, plain stores
        g.out = g.splitk_partials + (size_t)ks * g.M * g.N;
        g.epilogue = kEpiPartial;
        g.bias = nullptr;
    }

    uint32_t off[LPW];
    {
        const int rsub = 16 * wave + (lane >> 2);
        const int c = (lane & 3) ^ ((rsub >> 2) & 3);            // 128 i does not change (r / 4) % 4
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int r = rsub + 128 * i;
            const int row = (i < LPW_A) ? min(m0 + r, g.M - 1) : min(n0 + r - BM, g.N - 1);
            off[i] = (uint32_t)row * (uint32_t)g.K * 2u + (uint32_t)c * 16u;
        }
    }
    const unsigned char* a_base = reinterpret_cast<const unsigned char*>(g.a) + (size_t)kt0 * (BK * 2);
    const unsigned char* w_base = reinterpret_cast<const unsigned char*>(g.w) + (size_t)kt0 * (BK * 2);
    // load i of tile kt (clamped: past the end the last tile is fetched again into a stage nobody reads) into
    // the stage of iteration index st
    auto issue_load = [&](auto ic, int kt, int st) {
        constexpr int i = decltype(ic)::value;
        unsigned char* dst = smem_raw + (st & (NS - 1)) * STAGE_BYTES + (wave + NW * i) * 1024;
        load_to_lds_b128((i < LPW_A ? a_base : w_base) + (size_t)kt * (BK * 2) + off[i], dst);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int a_row0 = wm * (32 * TM) + l31;
    const int b_row0 = BM + wn * (32 * TN) + l31;
    bf16x8 fa[2][TM], fb[2][TN];
    auto read_step = [&](auto sc, int kt) {
        constexpr int s = decltype(sc)::value;
        const bf16* st = reinterpret_cast<const bf16*>(smem_raw + (kt & (NS - 1)) * STAGE_BYTES);
        const int coff = ((2 * s + lh) ^ ((l31 >> 2) & 3)) << 3;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[s][i] = *reinterpret_cast<const bf16x8*>(st + (a_row0 + 32 * i) * BK + coff);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[s][j] = *reinterpret_cast<const bf16x8*>(st + (b_row0 + 32 * j) * BK + coff);
    };
    auto mfma_step = [&](auto sc) {
        constexpr int s = decltype(sc)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s][i], fb[s][j], acc[i][j], 0, 0, 0);
    };
    // half an iteration: TM TN MFMAs, TM + TN fragment reads among the first of them, two loads at a quarter and
    // three quarters
    auto order_half = [&]() {
        constexpr int kM = TM * TN;
#pragma unroll
        for (int m = 0; m < kM; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (m < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (m == kM / 4 || m == 3 * kM / 4) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
    };
    auto barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    const std::integral_constant<int, 0> c0;
    const std::integral_constant<int, 1> c1;
    const std::integral_constant<int, 2> c2;
    const std::integral_constant<int, 3> c3;
    for (int p = 0; p < 3; ++p) {
        const int kt = min(p, nk - 1);
        issue_load(c0, kt, p);
        issue_load(c1, kt, p);
        issue_load(c2, kt, p);
        issue_load(c3, kt, p);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(LPW));      // tiles 0 and 1 have landed
    barrier();
    read_step(c0, 0);
    for (int kt = 0; kt < nk; ++kt) {
        const int lt = min(kt + 3, nk - 1);
        __builtin_amdgcn_sched_barrier(0);
        issue_load(c0, lt, kt + 3);
        issue_load(c1, lt, kt + 3);
        read_step(c1, kt);
        mfma_step(c0);
        order_half();
        __builtin_amdgcn_sched_barrier(0);
        issue_load(c2, lt, kt + 3);
        issue_load(c3, lt, kt + 3);
        read_step(c0, min(kt + 1, nk - 1));
        mfma_step(c1);
        order_half();
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(LPW));   // all but the newest tile's loads have landed
        barrier();
    }

    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    float* stage = reinterpret_cast<float*>(smem_raw) + wave * EPI_WAVE_FLOATS;
    run_epilogue<TM, TN>(g, acc, stage, m0 + wm * (32 * TM), n0 + wn * (32 * TN), lane);
}

// ---------------------------------------------------------------------------------------------------
// Alternating kernel for shapes that fill the chip with 256 x 256 tiles.  The eight waves work as two groups of
// four (one wave of each group on every SIMD) that run half a step apart.  A step of a wave is a memory phase (all
// fragment reads of the step, its share of the direct loads, then the waits) and a matrix phase (nothing but the
// step's 16 MFMAs), each closed by a workgroup barrier; group 1 takes one extra barrier before its first step and
// group 0 one after its last, so while one wave of a SIMD issues MFMAs back to back the other one reads LDS and
// waits, and the matrix pipe does not drain at a barrier that both of its waves reach together.
//   Rows are fetched in whole 128-byte lines (k tiles of 64).  A stage of 64 k is 64 KB and the LDS holds two and a
// half, so the ring is kept in half stages of 32 KB: unit 2t = the 256 rows of A for k tile t, unit 2t + 1 = the
// 256 rows of W, unit u in slot u % 5.  A step is half a k tile (two MFMA k steps); step 2t + h reads its fragments
// from the slots of units 2t and 2t + 1 at column half h and issues the loads of unit 2t + h + 3 into the slot that
// unit 2t + h - 2 left.
//   Barrier j (counted after the prologue's) closes the memory phase of step c for group 0 when j = 2c + 1, for
//   group 1 when j = 2c + 2.  Units 2t + 2 and 2t + 3 are first read in step 2t + 2, i.e. after barrier 4t + 4;
//   every wave waits for its own loads of both at the end of its memory phase of step 2t + 1 (only the loads of
//   unit 2t + 4 may still be in flight), i.e. before barrier 4t + 4 at the latest.  The slot of unit u - 5 was last
//   read in the memory phase of step u - 4 or u - 5 (the odd step of its tile) by group 1, which waits for its
//   fragments before the barrier that closes that phase; the loads of unit u are issued in step u - 3, after it.
//   Measured with s_memtime on one wave of each group (8192^3, clocks per step of 32 k; the step's MFMAs alone
// are 1030 per SIMD): fragment reads 250, direct loads 400, waits and barrier 100 = a memory phase of 750 against
// a matrix phase of 515, so a step takes 2 x 750.  What fills the memory phase is the LDS pipeline: about 5 clocks per
// ds_read_b128 of a wave and 25 per direct load here (alone on a compute unit a kilobyte takes 4.6 clocks to read,
// 16 to load directly and 13 to write with ds_write_b128: the rate microkernel of peaks.hip), whichever order the
// two are issued in and however far ahead the loads run (neither the latency of the loads nor the L2 is the limit:
// the same clocks per step with 16 workgroups and with 256, where the core clock drops from 2.4 to 1.8 GHz).
// Tried on this structure and dropped, all within the run-to-run spread of the figure above or worse: k tiles of 32
// in four or five stages (same clocks per step); reads and loads interleaved three to one, or half of the waves
// loading first (memory phase 740 to 770); the units staged through registers (global -> registers in the matrix
// phase, ds_write_b128 in the memory phase: memory phase 680; with the writes in the matrix phase too the MFMA
// wave stalls behind the other group's reads and a step grows by a fifth).
template <int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(512, 1) void gemm_alt64_kernel(GemmArgs g, int tiles_m, int tiles_n, int group_m,
                                                             int splitk) {
    static_assert(WM * WN == 8 && 32 * TM * WM == 256 && 32 * TN * WN == 256, "eight waves, 256 x 256 tiles");
    constexpr int NW = 8, BK = 64, SLOTS = 5, LPW = 4;
    constexpr int BM = 256;
    constexpr int UNIT_BYTES = 256 * BK * 2;         // 32 KB
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN;
    const int wn = wave % WN;
    const int l31 = lane & 31;
    const int lh = lane >> 5;

    const int nwg = gridDim.x;
    const int logical = (blockIdx.x & 7) * (nwg >> 3) + (blockIdx.x >> 3);
    const int tiles = tiles_m * tiles_n;
    if (logical >= tiles * splitk) return;
    const int ks = logical / tiles;                              // which part of k (0 when k is not split)
    const int t_id = logical - ks * tiles;
    const int group_size = group_m * tiles_n;
    const int grp = t_id / group_size;
    const int first_m = grp * group_m;
    const int gm = min(tiles_m - first_m, group_m);
    const int in_grp = t_id - grp * group_size;
    const int tile_m = first_m + in_grp % gm;
    const int tile_n = in_grp / gm;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * 256;
    const int nt_all = g.K / BK;
    const int kt0 = (int)((long long)ks * nt_all / splitk);
    const int nt = (int)((long long)(ks + 1) * nt_all / splitk) - kt0;
    if (splitk > 1) {                                            // this part's fp32 partial sums, plain stores
        g.out = g.splitk_partials + (size_t)ks * g.M * g.N;
        g.epilogue = kEpiPartial;
        g.bias = nullptr;
    }

    // A wave load fills 8 rows of 128 bytes; the lane that fills chunk position p of row r fetches logical chunk
    // p ^ ((r / 2) % 8) of that row (the swizzle of gemm_dma_kernel).
    uint32_t off_a[LPW], off_b[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int r = 8 * (wave + NW * i) + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        off_a[i] = (uint32_t)min(m0 + r, g.M - 1) * (uint32_t)g.K * 2u + (uint32_t)c * 16u;
        off_b[i] = (uint32_t)min(n0 + r, g.N - 1) * (uint32_t)g.K * 2u + (uint32_t)c * 16u;
    }
    const unsigned char* a_base = reinterpret_cast<const unsigned char*>(g.a) + (size_t)kt0 * (BK * 2);
    const unsigned char* w_base = reinterpret_cast<const unsigned char*>(g.w) + (size_t)kt0 * (BK * 2);
    // the rows of A (of W) for k tile t, clamped (past the end the last tile is fetched again into a slot nobody reads)
    auto issue_a = [&](int t, int slot) {
        const unsigned char* src = a_base + (size_t)min(t, nt - 1) * (BK * 2);
        unsigned char* dst = smem_raw + slot * UNIT_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < LPW; ++i) load_to_lds_b128(src + off_a[i], dst + i * (NW * 1024));
    };
    auto issue_b = [&](int t, int slot) {
        const unsigned char* src = w_base + (size_t)min(t, nt - 1) * (BK * 2);
        unsigned char* dst = smem_raw + slot * UNIT_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < LPW; ++i) load_to_lds_b128(src + off_b[i], dst + i * (NW * 1024));
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int a_row0 = wm * (32 * TM) + l31;
    const int b_row0 = wn * (32 * TN) + l31;
    const int key = (l31 >> 1) & 7;
    bf16x8 fa[2][TM], fb[2][TN];
    // fragments of the two MFMA k steps of column half h
    auto read_half = [&](auto hc, int slot_a, int slot_b) {
        constexpr int h = decltype(hc)::value;
        const bf16* sa = reinterpret_cast<const bf16*>(smem_raw + slot_a * UNIT_BYTES);
        const bf16* sb = reinterpret_cast<const bf16*>(smem_raw + slot_b * UNIT_BYTES);
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const int coff = ((2 * (2 * h + s2) + lh) ^ key) << 3;
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[s2][i] = *reinterpret_cast<const bf16x8*>(sa + (a_row0 + 32 * i) * BK + coff);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[s2][j] = *reinterpret_cast<const bf16x8*>(sb + (b_row0 + 32 * j) * BK + coff);
        }
    };
    auto mfma_half = [&]() {
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s2][i], fb[s2][j], acc[i][j], 0, 0, 0);
    };
    auto barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    auto next = [](int slot, int by) { return slot + by >= SLOTS ? slot + by - SLOTS : slot + by; };

    const std::integral_constant<int, 0> h0;
    const std::integral_constant<int, 1> h1;
    const bool second_group = wave >= NW / 2;        // wave-uniform (wave is in a scalar register)
    issue_a(0, 0);
    issue_b(0, 1);
    issue_a(1, 2);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(LPW));      // units 0 and 1 have landed
    barrier();
    if (second_group) barrier();
    int sa = 0, sb = 1, sl = 3;                      // slots of A and W of tile t, slot of the next unit to load
    for (int t = 0; t < nt; ++t) {
        // ---- step 2t, memory phase: fragments of the first column half, loads of unit 2t + 3 (W of tile t + 1)
        __builtin_amdgcn_sched_barrier(0);
        read_half(h0, sa, sb);
        issue_b(t + 1, sl);
        sl = next(sl, 1);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0xC07F);          // the fragments are in registers (lgkmcnt 0, no wait on loads)
        barrier();
        __builtin_amdgcn_sched_barrier(0);
        mfma_half();
        __builtin_amdgcn_sched_barrier(0);
        barrier();
        // ---- step 2t + 1: second column half, loads of unit 2t + 4 (A of tile t + 2); tile t + 1 has landed
        __builtin_amdgcn_sched_barrier(0);
        read_half(h1, sa, sb);
        issue_a(t + 2, sl);
        sl = next(sl, 1);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(LPW) & 0xF0FF);
        barrier();
        __builtin_amdgcn_sched_barrier(0);
        mfma_half();
        __builtin_amdgcn_sched_barrier(0);
        barrier();
        sa = next(sa, 2);
        sb = next(sb, 2);
    }
    if (!second_group) barrier();

    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    float* stage = reinterpret_cast<float*>(smem_raw) + wave * EPI_WAVE_FLOATS;
    run_epilogue<TM, TN>(g, acc, stage, m0 + wm * (32 * TM), n0 + wn * (32 * TN), lane);
}

template <int WM, int WN, int TM, int TN>
hipError_t launch_ring(const GemmArgs& g, int splitk, hipStream_t s) {
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    constexpr size_t smem = (size_t)4 * (BM + BN) * 32 * sizeof(bf16);
    static_assert(smem <= 160 * 1024 && smem >= (size_t)8 * EPI_WAVE_FLOATS * sizeof(float), "LDS");
    const int tiles_m = (g.M + BM - 1) / BM;
    const int tiles_n = (g.N + BN - 1) / BN;
    const int grid = (tiles_m * tiles_n * splitk + 7) / 8 * 8;
    static std::once_flag attr_once;          // one per instantiation
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&]() {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_ring_kernel<WM, WN, TM, TN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    });
    if (attr_err != hipSuccess || attributes_only()) return attr_err;
    // groups of four tile rows: an XCD's 32 concurrent tiles then cover 4 x 8 tiles, the shape with the fewest
    // distinct operand rows per k step
    hipLaunchKernelGGL((gemm_ring_kernel<WM, WN, TM, TN>), dim3(grid), dim3(512), smem, s, g, tiles_m, tiles_n, 4, splitk);
    return hipGetLastError();
}

template <int WM, int WN, int TM, int TN>
hipError_t launch_alt64(const GemmArgs& g, int splitk, hipStream_t s) {
    constexpr size_t smem = (size_t)5 * 256 * 64 * sizeof(bf16);      // five half stages: all 160 KB
    static_assert(smem <= 160 * 1024 && smem >= (size_t)8 * EPI_WAVE_FLOATS * sizeof(float), "LDS");
    const int tiles_m = (g.M + 255) / 256;
    const int tiles_n = (g.N + 255) / 256;
    const int grid = (tiles_m * tiles_n * splitk + 7) / 8 * 8;
    static std::once_flag attr_once;          // one per instantiation
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&]() {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_alt64_kernel<WM, WN, TM, TN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    });
    if (attr_err != hipSuccess || attributes_only()) return attr_err;
    hipLaunchKernelGGL((gemm_alt64_kernel<WM, WN, TM, TN>), dim3(grid), dim3(512), smem, s, g, tiles_m, tiles_n, 4, splitk);
    return hipGetLastError();
}

template <int WM, int WN, int TM, int TN, int NS>
hipError_t launch_dma(const GemmArgs& g, int splitk, hipStream_t s) {
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    constexpr size_t smem = (size_t)NS * (BM + BN) * 64 * sizeof(bf16);
    static_assert(smem <= 160 * 1024, "LDS stages exceed 160 KB");
    static_assert(smem >= (size_t)WM * WN * EPI_WAVE_FLOATS * sizeof(float), "epilogue staging");
    const int tiles_m = (g.M + BM - 1) / BM;
    const int tiles_n = (g.N + BN - 1) / BN;
    const int grid = (tiles_m * tiles_n * splitk + 7) / 8 * 8;
    static std::once_flag attr_once;          // one per instantiation
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&]() {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_kernel<WM, WN, TM, TN, NS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    });
    if (attr_err != hipSuccess || attributes_only()) return attr_err;
    const int group_m = (32 * TM * WM >= 256) ? 4 : 8;
    hipLaunchKernelGGL((gemm_dma_kernel<WM, WN, TM, TN, NS>), dim3(grid), dim3(64 * WM * WN), smem, s, g, tiles_m, tiles_n,
                       group_m, splitk);
    return hipGetLastError();
}

struct TilePlan {
    int tm, tn, pf;       // register-staged kernel: tile (128 tm) x (32 tn), pf register sets
    int dma = 0;          // otherwise: a configuration of the direct-load kernel (tm, tn, pf unused)
    int splitk = 1;       // register-staged kernel: parts of the k range, each its own workgroup (needs scratch)
};

// Tile plans measured on MI355X for the projection shapes of the 1.3B- and 14B-shaped blocks with a
// 1024-token chunk (sweep over every (TM, TN, PF) of the register-staged kernel and every configuration of
// the direct-load kernel).
struct TunedShape {
    int M, N, K;
    TilePlan plan;
};
const TunedShape kTuned[] = {
    // the 1.3B block on one 1024-token chunk, weights cold (every launch of the sweep reads another copy): small
    // tiles of the direct-load kernel are 2 to 12 % faster than the register-staged kernel's best
    {1024, 4608, 1536, {0, 0, 0, 16}},         // QKV: 128 x 192, eight waves
    {1024, 1536, 1536, {0, 0, 0, 9}},          // C x C projections: 128 x 64, eight waves of 32 x 32
    {1024, 8960, 1536, {0, 0, 0, 13}},         // FFN-1: 128 x 160, two stages, two workgroups per unit
    {1024, 1536, 8960, {0, 0, 0, 16, 4}},      // FFN-2: 128 x 192, four k parts
    {1024, 5120, 5120, {1, 5, 2}},  {1024, 5120, 13824, {0, 0, 0, 5, 3}},      // FFN-2 14B: ring, 256 x 256 tiles, three k parts
    // the 1.3B block with 2 or 4 streams per call, where the rule below is more than 4 % off the sweep's best
    {2048, 1536, 8960, {1, 6, 2, 0, 2}}, {4096, 8960, 1536, {1, 5, 2}}, {4096, 1536, 8960, {1, 6, 2}},
    {4096, 1536, 1536, {0, 0, 0, 16}}, {4096, 4608, 1536, {0, 0, 0, 16}},
};

// Otherwise: when 256 x 256 tiles fill at least 80 % of the compute units in every round, the direct-load
// kernel with that tile wins (it moves the fewest bytes per flop through the LDS and the L2), in its alternating
// variant (+6 to +9 % over the ring variant on the batched 480p shapes, equal within 2 % on the 1024-row shapes of the
// 14B block; the ring variant is +2 to +15 % over the two-stage one).  Else estimate the time of the busiest compute unit for the register-staged kernel: one k
// tile of a workgroup costs a fixed part (~0.25 us alone, half of it when a second workgroup fills the
// bubbles) plus ~21 ns per MFMA a wave issues (fitted to the sweep); small tiles fit two workgroups per unit.
// The direct-load kernels address an operand with 32-bit byte offsets per lane: they serve operands below 4 GiB.
bool fits_32bit_offsets(int M, int N, int K) {
    return (unsigned long long)M * K * 2 <= 0xFFFFFFFFull && (unsigned long long)N * K * 2 <= 0xFFFFFFFFull;
}

TilePlan plan_tiles(int M, int N, int K, int epilogue) {
    (void)epilogue;
    const bool direct_ok = fits_32bit_offsets(M, N, K);
    for (const TunedShape& t : kTuned)
        if (t.M == M && t.N == N && t.K == K && (direct_ok || !t.plan.dma)) return t.plan;
    const int kCUs = 256;
    if (direct_ok) {
        const long long tiles = (long long)((M + 255) / 256) * ((N + 255) / 256);
        const long long rounds = (tiles + kCUs - 1) / kCUs;
        if (K >= 512 && tiles * 10 >= rounds * kCUs * 8) return TilePlan{0, 0, 0, 18};
    }
    TilePlan best{1, 4, 2};
    double best_cost = 1e300;
    for (int tm = 1; tm <= 2; ++tm) {
        for (int tn = 2; tn <= 7; ++tn) {
            const int wgs = ((M + 128 * tm - 1) / (128 * tm)) * ((N + 32 * tn - 1) / (32 * tn));
            const int occ = (tm * tn <= 5) ? 2 : 1;
            const int per_cu = (wgs + kCUs - 1) / kCUs;
            const double mfma = 0.021 * 4 * tm * tn;
            double cost;
            if (occ == 2 && per_cu >= 2) cost = (per_cu + 1) / 2 * (0.25 + 2 * mfma);
            else cost = per_cu * (0.25 + mfma);
            cost = cost * (K / 64) + per_cu * 0.04 * tm * tn;      // + epilogue
            if (cost < best_cost) {
                best_cost = cost;
                best = TilePlan{tm, tn, 2};
            }
        }
    }
    return best;
}

template <int TM, int TN, int PF>
hipError_t launch_one(const GemmArgs& g, int splitk, hipStream_t s) {
    constexpr int BK = 64;
    constexpr int BM = 128 * TM, BN = 32 * TN;
    const int tiles_m = (g.M + BM - 1) / BM;
    const int tiles_n = (g.N + BN - 1) / BN;
    const int grid = (tiles_m * tiles_n * splitk + 7) / 8 * 8;
    const size_t smem = (size_t)2 * (BM + BN) * BK * sizeof(bf16);
    static_assert((size_t)2 * (BM + BN) * BK * sizeof(bf16) >= 4 * EPI_WAVE_FLOATS * sizeof(float), "epilogue staging");
    static std::once_flag attr_once;          // one per instantiation
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&]() {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<TM, TN, BK, PF>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    });
    if (attr_err != hipSuccess || attributes_only()) return attr_err;
    const int group_m = 8;
    hipLaunchKernelGGL((gemm_kernel<TM, TN, BK, PF>), dim3(grid), dim3(256), smem, s, g, tiles_m, tiles_n, group_m, splitk);
    return hipGetLastError();
}

template <int TM, int PF>
hipError_t launch_tn(const GemmArgs& g, int tn, int splitk, hipStream_t s) {
    switch (tn) {
        case 2: return launch_one<TM, 2, PF>(g, splitk, s);
        case 3: return launch_one<TM, 3, PF>(g, splitk, s);
        case 4: return launch_one<TM, 4, PF>(g, splitk, s);
        case 5: return launch_one<TM, 5, PF>(g, splitk, s);
        case 6: return launch_one<TM, 6, PF>(g, splitk, s);
    }
    if constexpr (PF == 2) {
        switch (tn) {
            case 7: return launch_one<TM, 7, PF>(g, splitk, s);
            case 8: return launch_one<TM, 8, PF>(g, splitk, s);
        }
    }
    return hipErrorInvalidValue;
}

// Configurations of the direct-load kernel: (waves on M, waves on N, TM, TN, LDS stages).  Ids 1-6 are the large
// tiles for shapes that fill the chip; ids 7 and up are small tiles for the skinny shapes of a single 1024-token
// chunk, where the tile count has to reach the number of compute units and a k iteration holds only a few matrix
// instructions per wave: no staging registers and no LDS write instructions, three or four tiles in flight, and
// two or three workgroups per compute unit to cover the barrier.
constexpr int kDmaConfigs = 18;
hipError_t launch_dma_config(const GemmArgs& g, int id, int splitk, hipStream_t s) {
    if (!fits_32bit_offsets(g.M, g.N, g.K)) return hipErrorInvalidValue;     // only reachable through the tuning override
    switch (id) {
        case 1: return launch_dma<4, 2, 2, 4, 2>(g, splitk, s);      // 256 x 256, wave tile 64 x 128
        case 2: return launch_dma<2, 4, 4, 2, 2>(g, splitk, s);      // 256 x 256, wave tile 128 x 64
        case 3: return launch_dma<2, 4, 2, 2, 3>(g, splitk, s);      // 128 x 256
        case 4: return launch_dma<4, 2, 2, 2, 3>(g, splitk, s);      // 256 x 128
        case 5: return launch_ring<4, 2, 2, 4>(g, splitk, s);        // 256 x 256, ring of four k32 stages
        case 6: return launch_ring<2, 4, 4, 2>(g, splitk, s);
        case 7: return launch_dma<4, 1, 1, 2, 3>(g, splitk, s);      // 128 x 64, four waves, 72 KB: two workgroups per unit
        case 8: return launch_dma<4, 1, 1, 2, 4>(g, splitk, s);      // 128 x 64, four stages
        case 9: return launch_dma<4, 2, 1, 1, 4>(g, splitk, s);      // 128 x 64, eight waves of 32 x 32
        case 10: return launch_dma<2, 2, 1, 2, 4>(g, splitk, s);     // 64 x 128, four waves
        case 11: return launch_dma<2, 2, 2, 2, 3>(g, splitk, s);     // 128 x 128, four waves of 64 x 64
        case 12: return launch_dma<2, 4, 2, 1, 3>(g, splitk, s);     // 128 x 128, eight waves of 64 x 32
        case 13: return launch_dma<4, 1, 1, 5, 2>(g, splitk, s);     // 128 x 160, four waves, two stages (72 KB)
        case 14: return launch_dma<4, 1, 1, 5, 3>(g, splitk, s);     // 128 x 160, three stages
        case 15: return launch_dma<4, 1, 1, 6, 3>(g, splitk, s);     // 128 x 192
        case 16: return launch_dma<4, 2, 1, 3, 3>(g, splitk, s);     // 128 x 192, eight waves of 32 x 96
        case 17: return launch_alt64<4, 2, 2, 4>(g, splitk, s);      // 256 x 256, two wave groups half a step apart, ring of five half stages
        case 18: return launch_alt64<2, 4, 4, 2>(g, splitk, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

// Plan override for tuning runs and tests, set through sdv2_tuning_set("gemm_tile", ...): "tm,tn[,pf[,splitk]]"
// picks a tile of the register-staged kernel, "d<id>[,splitk]" a configuration of the direct-load kernel; an empty
// string or null clears it.  Not read from the environment: a production
// process cannot change a kernel plan by accident, and a launch costs no getenv.
static bool g_have_tile_override = false;
static TilePlan g_tile_override;

bool set_gemm_tile_override(const char* e) {
    if (!e || !*e) {
        g_have_tile_override = false;
        return true;
    }
    int a, b, d = 2;
    int dk = 1;
    if (sscanf(e, "d%d,%d", &a, &dk) >= 1 && a >= 1 && a <= kDmaConfigs && dk >= 1 && dk <= 16) {
        g_tile_override = TilePlan{0, 0, 0, a, dk};
        g_have_tile_override = true;
        return true;
    }
    int k = 1;
    if (sscanf(e, "%d,%d,%d,%d", &a, &b, &d, &k) >= 2 && a >= 1 && a <= 2 && b >= 2 && b <= 8 &&
        (d == 2 || (d == 3 && b <= 6)) && k >= 1 && k <= 8) {
        g_tile_override = TilePlan{a, b, d, 0, k};
        g_have_tile_override = true;
        return true;
    }
    return false;
}

static thread_local bool g_attr_only = false;
void set_attributes_only(bool on) { g_attr_only = on; }
bool attributes_only() { return g_attr_only; }

static bool tile_override(TilePlan* p) {
    if (g_have_tile_override) *p = g_tile_override;
    return g_have_tile_override;
}

namespace {
// out = epilogue(sum of the k parts + bias), four columns per thread; the parts are added in k order.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmArgs g, int splitk) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // over M * N / 4
    const size_t n4 = (size_t)(g.N >> 2);
    if (idx >= (size_t)g.M * n4) return;
    const int row = (int)(idx / n4);
    const int col = (int)(idx - (size_t)row * n4) * 4;
    const size_t o = (size_t)row * g.N + col;
    const size_t part = (size_t)g.M * g.N;
    f32x4 v = *reinterpret_cast<const f32x4*>(g.splitk_partials + o);
    for (int s = 1; s < splitk; ++s) v += *reinterpret_cast<const f32x4*>(g.splitk_partials + s * part + o);
    if (g.bias != nullptr) v += *reinterpret_cast<const f32x4*>(g.bias + col);
    if (g.epilogue == kEpiBias || g.epilogue == kEpiBiasGelu) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (bf16)(g.epilogue == kEpiBiasGelu ? gelu_tanh_f(v[e]) : v[e]);
        *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16*>(g.out) + o) = w;
    } else {
        if (g.epilogue == kEpiGatedResidual) {
            const f32x4 ga = *reinterpret_cast<const f32x4*>(g.gate_a + col);
            const f32x4 gb = *reinterpret_cast<const f32x4*>(g.gate_b + (size_t)(row / g.rows_per_gate) * g.gate_b_stride + col);
            v *= (ga + gb);
        }
        float* xo = reinterpret_cast<float*>(g.out) + o;
        *reinterpret_cast<f32x4*>(xo) = *reinterpret_cast<const f32x4*>(xo) + v;
    }
}
}  // namespace

namespace {
// The same sum of the k parts for a residual epilogue whose result is LayerNorm-ed next: a workgroup of four waves
// owns a row, adds the parts in k order, applies bias, gate and residual, stores the new fp32 row, and normalises it
// from the registers: one launch and one read of x less than reduce + LayerNorm.  (One row per workgroup: the pass
// reads splitk + 1 fp32 rows per output row, and with fewer, fatter workgroups it ran at 2.5 TB/s.)
template <int NV>
__global__ __launch_bounds__(256) void splitk_reduce_ln_kernel(GemmArgs g, int splitk, LnArgs ln) {
    __shared__ float part[4][2];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t = threadIdx.x;
    const int row = blockIdx.x;
    const int nvec = g.N >> 2;
    const size_t plane = (size_t)g.M * g.N;
    float* xrow = reinterpret_cast<float*>(g.out) + (size_t)row * g.N;
    const float* prow = g.splitk_partials + (size_t)row * g.N;
    const int stream = row / g.rows_per_gate;
    const int ln_stream = row / ln.rows_per_stream;
    const float pivot = xrow[0];                          // any value near the row's mean: read before the row is rewritten
    f32x4 v[NV], sc[NV], sh[NV];
    // everything the row needs is requested at once: the parts, x, bias and gate, and the LayerNorm's scale and shift
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = t + 256 * i;
        if (idx < nvec) {
            const int c = idx * 4;
            f32x4 acc = *reinterpret_cast<const f32x4*>(prow + c);
            for (int sp = 1; sp < splitk; ++sp) acc += *reinterpret_cast<const f32x4*>(prow + sp * plane + c);
            if (g.bias != nullptr) acc += *reinterpret_cast<const f32x4*>(g.bias + c);
            if (g.epilogue == kEpiGatedResidual)
                acc *= *reinterpret_cast<const f32x4*>(g.gate_a + c) +
                       *reinterpret_cast<const f32x4*>(g.gate_b + (size_t)stream * g.gate_b_stride + c);
            v[i] = *reinterpret_cast<const f32x4*>(xrow + c) + acc;
            sc[i] = *reinterpret_cast<const f32x4*>(ln.scale_a + c);
            sh[i] = *reinterpret_cast<const f32x4*>(ln.shift_a + c);
            if (ln.scale_b != nullptr) {
                sc[i] += *reinterpret_cast<const f32x4*>(ln.scale_b + (size_t)ln_stream * ln.b_stride + c);
                sh[i] += *reinterpret_cast<const f32x4*>(ln.shift_b + (size_t)ln_stream * ln.b_stride + c);
                sc[i] += 1.0f;
            }
        }
    }
    __syncthreads();                                      // every thread of the row has read the pivot before x changes
    float sum = 0.0f, sq = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = t + 256 * i;
        if (idx < nvec) {
            *reinterpret_cast<f32x4*>(xrow + idx * 4) = v[i];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float d = v[i][e] - pivot;
                sum += d;
                sq += d * d;
            }
        }
    }
    sum = wave_sum(sum);
    sq = wave_sum(sq);
    if (lane == 0) {
        part[wave][0] = sum;
        part[wave][1] = sq;
    }
    __syncthreads();
    sum = (part[0][0] + part[1][0]) + (part[2][0] + part[3][0]);
    sq = (part[0][1] + part[1][1]) + (part[2][1] + part[3][1]);
    const float inv_c = 1.0f / (float)g.N;
    const float dmean = sum * inv_c;
    const float var = fmaxf(sq * inv_c - dmean * dmean, 0.0f);
    const float rstd = rsqrtf(var + ln.eps);
    const float mean = pivot + dmean;
    bf16* op = ln.out + (size_t)row * g.N;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = t + 256 * i;
        if (idx < nvec) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)((v[i][e] - mean) * rstd * sc[i][e] + sh[i][e]);
            *reinterpret_cast<bf16x4*>(op + idx * 4) = o;
        }
    }
}
}  // namespace

// Parts of k the plan can really use for this problem and scratch (1: no split).
static int usable_splitk(const GemmArgs& g, const TilePlan& p) {
    if (p.splitk <= 1 || g.splitk_partials == nullptr) return 1;
    int splitk = p.splitk;
    if (splitk > g.K / 128) splitk = g.K / 128;                 // at least two k tiles per part
    if (splitk < 2 || (size_t)splitk * g.M * g.N > g.splitk_floats) return 1;
    return splitk;
}

// part 0: the whole product; 1: only the kernel on the matrix cores; 2: only the pass that adds the k parts (nothing
// when the plan does not split).  The benchmark times the two parts separately.
static hipError_t launch_gemm_impl(const GemmArgs& g, const LnArgs* ln, bool* ln_done, hipStream_t s, int part = 0) {
    TilePlan p = plan_tiles(g.M, g.N, g.K, g.epilogue);
    tile_override(&p);
    const int splitk = usable_splitk(g, p);
    hipError_t e = hipSuccess;
    if (part != 2) {
        if (p.dma) e = launch_dma_config(g, p.dma, splitk, s);
        else if (p.pf == 3) e = p.tm == 1 ? launch_tn<1, 3>(g, p.tn, splitk, s) : launch_tn<2, 3>(g, p.tn, splitk, s);
        else e = p.tm == 1 ? launch_tn<1, 2>(g, p.tn, splitk, s) : launch_tn<2, 2>(g, p.tn, splitk, s);
    }
    if (e != hipSuccess || splitk == 1 || attributes_only() || part == 1) return e;
    const int nv = (g.N + 1023) / 1024;                 // float4 values per thread with 256 threads per row
    if (ln != nullptr && (g.epilogue == kEpiGatedResidual || g.epilogue == kEpiResidual) && nv <= 8) {
        const dim3 grid(g.M), block(256);
        if (nv <= 1) hipLaunchKernelGGL(splitk_reduce_ln_kernel<1>, grid, block, 0, s, g, splitk, *ln);
        else if (nv <= 2) hipLaunchKernelGGL(splitk_reduce_ln_kernel<2>, grid, block, 0, s, g, splitk, *ln);
        else if (nv <= 3) hipLaunchKernelGGL(splitk_reduce_ln_kernel<3>, grid, block, 0, s, g, splitk, *ln);
        else if (nv <= 5) hipLaunchKernelGGL(splitk_reduce_ln_kernel<5>, grid, block, 0, s, g, splitk, *ln);
        else hipLaunchKernelGGL(splitk_reduce_ln_kernel<8>, grid, block, 0, s, g, splitk, *ln);
        *ln_done = true;
        return hipGetLastError();
    }
    const size_t n = (size_t)g.M * (g.N >> 2);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, g, splitk);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) { return launch_gemm_impl(g, nullptr, nullptr, s); }

// Name of the kernel instantiation the plan picks for a shape, spelled as a profiler prints it.
void gemm_plan_name(int M, int N, int K, int epilogue, char* out, size_t cap) {
    TilePlan p = plan_tiles(M, N, K, epilogue);
    tile_override(&p);
    static const int kDma[kDmaConfigs + 1][5] = {{0, 0, 0, 0, 0}, {4, 2, 2, 4, 2}, {2, 4, 4, 2, 2}, {2, 4, 2, 2, 3}, {4, 2, 2, 2, 3},
                                                 {4, 2, 2, 4, 0}, {2, 4, 4, 2, 0}, {4, 1, 1, 2, 3}, {4, 1, 1, 2, 4}, {4, 2, 1, 1, 4},
                                                 {2, 2, 1, 2, 4}, {2, 2, 2, 2, 3}, {2, 4, 2, 1, 3}, {4, 1, 1, 5, 2}, {4, 1, 1, 5, 3},
                                                 {4, 1, 1, 6, 3}, {4, 2, 1, 3, 3}, {4, 2, 2, 4, 0}, {2, 4, 4, 2, 0}};
    if (p.dma >= 17)
        snprintf(out, cap, "gemm_alt64_kernel<%d, %d, %d, %d>", kDma[p.dma][0], kDma[p.dma][1], kDma[p.dma][2], kDma[p.dma][3]);
    else if (p.dma == 5 || p.dma == 6)
        snprintf(out, cap, "gemm_ring_kernel<%d, %d, %d, %d>", kDma[p.dma][0], kDma[p.dma][1], kDma[p.dma][2], kDma[p.dma][3]);
    else if (p.dma)
        snprintf(out, cap, "gemm_dma_kernel<%d, %d, %d, %d, %d>", kDma[p.dma][0], kDma[p.dma][1], kDma[p.dma][2], kDma[p.dma][3],
                 kDma[p.dma][4]);
    else
        snprintf(out, cap, "gemm_kernel<%d, %d, 64, %d>", p.tm, p.tn, p.pf);
}

hipError_t launch_gemm_then_layernorm(const GemmArgs& g, const LnArgs& ln, bool* ln_done, hipStream_t s, int part) {
    *ln_done = false;
    return launch_gemm_impl(g, &ln, ln_done, s, part);
}

hipError_t launch_gemm_part(const GemmArgs& g, hipStream_t s, int part) { return launch_gemm_impl(g, nullptr, nullptr, s, part); }

bool gemm_splits_k(const GemmArgs& g) {
    TilePlan p = plan_tiles(g.M, g.N, g.K, g.epilogue);
    tile_override(&p);
    return usable_splitk(g, p) > 1;
}

size_t gemm_splitk_floats(int M, int N, int K, int epilogue) {
    TilePlan p = plan_tiles(M, N, K, epilogue);
    tile_override(&p);
    if (p.splitk <= 1) return 0;
    return (size_t)p.splitk * M * N;
}

}  // namespace sdv2

