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
//   * Tiles go global -> registers -> LDS, double buffered, one barrier per k tile.  LDS rows are
//     64 bf16 (128 B); the 16-byte chunk index is XOR-ed with (row % 8) so that the 32 lanes of a
//     fragment read hit all banks.
//   * Workgroup ids are spread round-robin over the 8 XCDs by the hardware; the kernel undoes that
//     so that each XCD (one L2) owns a contiguous range of tiles, ordered in groups of M tiles that
//     share weight tiles.
//   * Optional split-K for the two fp32 read-modify-write epilogues (hardware fp32 atomics on x).
#include "common.h"

#include <stdio.h>
#include <stdlib.h>

namespace sdv2 {

namespace {

constexpr int BK = 64;

// Accumulator register r of a 32x32 block holds row 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32.
// row0 / col0 already contain the lane's 4 (lane / 32) and lane % 32.
template <int TM, int TN, int EPI>
__device__ __forceinline__ void epilogue(const GemmArgs& g, f32x16 (&acc)[TM][TN], int row0, int col0, bool lead,
                                         bool atomic) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = col0 + 32 * j;
        const bool col_ok = col < g.N;
        const int colc = col_ok ? col : 0;
        const float bias = (g.bias != nullptr && lead) ? g.bias[colc] : 0.0f;
        float gate_a = 0.0f;
        if (EPI == kEpiGatedResidual) gate_a = g.gate_a[colc];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row0 + 32 * i + 8 * (r >> 2) + (r & 3);
                if (col_ok && row < g.M) {
                    const float v = acc[i][j][r] + bias;
                    const size_t o = (size_t)row * g.N + col;
                    if (EPI == kEpiBias) {
                        reinterpret_cast<bf16*>(g.out)[o] = (bf16)v;
                    } else if (EPI == kEpiBiasGelu) {
                        reinterpret_cast<bf16*>(g.out)[o] = (bf16)gelu_tanh_f(v);
                    } else {
                        float add = v;
                        if (EPI == kEpiGatedResidual) {
                            const int sidx = row / g.rows_per_gate;
                            add = (gate_a + g.gate_b[(size_t)sidx * g.gate_b_stride + col]) * v;
                        }
                        float* xo = reinterpret_cast<float*>(g.out) + o;
                        if (atomic) {
                            unsafeAtomicAdd(xo, add);
                        } else {
                            *xo += add;
                        }
                    }
                }
            }
        }
    }
}

template <int TM, int TN>
__global__ __launch_bounds__(256, 1) void gemm_kernel(GemmArgs g, int tiles_m, int tiles_n, int group_m,
                                                      int splitk) {
    constexpr int BM = 128 * TM;
    constexpr int BN = 32 * TN;
    constexpr int NA = 4 * TM;      // 16-byte chunks of the A tile per thread
    constexpr int NB = TN;          // of the W tile
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* const sm = reinterpret_cast<bf16*>(smem_raw);     // [2][BM*64 | BN*64]
    constexpr int STAGE = (BM + BN) * BK;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l31 = lane & 31;
    const int lh = lane >> 5;
    const int l7 = lane & 7;

    // ---- which tile: undo the round-robin XCD dispatch, then grouped ordering
    const int nwg = gridDim.x;                                   // multiple of 8
    const int logical = (blockIdx.x & 7) * (nwg >> 3) + (blockIdx.x >> 3);
    const int tiles = tiles_m * tiles_n;
    if (logical >= tiles * splitk) return;
    const int ks = logical / tiles;
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

    // ---- global -> register staging
    const int crow = tid >> 3;          // 0..31
    const int cchunk = tid & 7;
    const bf16* ap[NA];
    const bf16* bp[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int row = min(m0 + crow + 32 * i, g.M - 1);
        ap[i] = g.a + (size_t)row * g.K + cchunk * 8;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int row = min(n0 + crow + 32 * i, g.N - 1);
        bp[i] = g.w + (size_t)row * g.K + cchunk * 8;
    }
    const int st_off = crow * BK + ((cchunk ^ (crow & 7)) << 3);
    bf16x8 ra[NA], rb[NB];

    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = *reinterpret_cast<const bf16x8*>(ap[i] + kt * BK);
#pragma unroll
        for (int i = 0; i < NB; ++i) rb[i] = *reinterpret_cast<const bf16x8*>(bp[i] + kt * BK);
    };
    auto sstore = [&](int buf) {
        bf16* sa = sm + buf * STAGE;
        bf16* sb = sa + BM * BK;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<bf16x8*>(sa + st_off + i * 32 * BK) = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *reinterpret_cast<bf16x8*>(sb + st_off + i * 32 * BK) = rb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int a_row0 = wave * (32 * TM) + l31;

    if (kt0 < kt1) {
        gload(kt0);
        sstore(0);
    }
    __syncthreads();
    for (int kt = kt0; kt < kt1; ++kt) {
        const int buf = (kt - kt0) & 1;
        if (kt + 1 < kt1) gload(kt + 1);
        const bf16* sa = sm + buf * STAGE;
        const bf16* sb = sa + BM * BK;
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const int coff = ((2 * s + lh) ^ l7) << 3;
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(sa + (a_row0 + 32 * i) * BK + coff);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(sb + (l31 + 32 * j) * BK + coff);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < kt1) sstore(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue
    const int row0 = m0 + wave * (32 * TM) + 4 * lh;
    const int col0 = n0 + l31;
    switch (g.epilogue) {
        case kEpiBias: epilogue<TM, TN, kEpiBias>(g, acc, row0, col0, ks == 0, splitk > 1); break;
        case kEpiBiasGelu: epilogue<TM, TN, kEpiBiasGelu>(g, acc, row0, col0, ks == 0, splitk > 1); break;
        case kEpiGatedResidual: epilogue<TM, TN, kEpiGatedResidual>(g, acc, row0, col0, ks == 0, splitk > 1); break;
        default: epilogue<TM, TN, kEpiResidual>(g, acc, row0, col0, ks == 0, splitk > 1); break;
    }
}

struct TilePlan {
    int tm, tn, splitk;
};

// Choose the tile so that the busiest compute unit finishes first.  cost(tile) is in units of
// "32x32x16 MFMA issue slots per k step", inflated by the LDS fragment traffic per MFMA, which is what
// separates a skinny tile from a square one.
TilePlan plan_tiles(int M, int N, int K, int epilogue) {
    const int kCUs = 256;
    TilePlan best{1, 4, 1};
    double best_cost = 1e300;
    const bool can_split = (epilogue == kEpiGatedResidual || epilogue == kEpiResidual);
    for (int tm = 1; tm <= 2; ++tm) {
        for (int tn = 2; tn <= 8; ++tn) {
            const int tiles = ((M + 128 * tm - 1) / (128 * tm)) * ((N + 32 * tn - 1) / (32 * tn));
            for (int sk = 1; sk <= (can_split ? 4 : 1); sk *= 2) {
                if ((K / BK) / sk < 8) continue;
                const int wgs = tiles * sk;
                const int per_cu = (wgs + kCUs - 1) / kCUs;
                const double frag_per_mfma = (double)(tm + tn) / (tm * tn);
                const double eff = 1.0 / (1.0 + 0.35 * frag_per_mfma);
                double cost = (double)per_cu * (tm * tn) * (K / BK / sk + 2) / eff;
                if (sk > 1) cost *= 1.05;       // atomics in the epilogue
                if (cost < best_cost) {
                    best_cost = cost;
                    best = TilePlan{tm, tn, sk};
                }
            }
        }
    }
    return best;
}

template <int TM, int TN>
hipError_t launch_one(const GemmArgs& g, int splitk, hipStream_t s) {
    constexpr int BM = 128 * TM, BN = 32 * TN;
    const int tiles_m = (g.M + BM - 1) / BM;
    const int tiles_n = (g.N + BN - 1) / BN;
    const int wgs = tiles_m * tiles_n * splitk;
    const int grid = (wgs + 7) / 8 * 8;
    const size_t smem = (size_t)2 * (BM + BN) * BK * sizeof(bf16);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<TM, TN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int group_m = 8;
    hipLaunchKernelGGL((gemm_kernel<TM, TN>), dim3(grid), dim3(256), smem, s, g, tiles_m, tiles_n, group_m,
                       splitk);
    return hipGetLastError();
}

template <int TM>
hipError_t launch_tn(const GemmArgs& g, int tn, int splitk, hipStream_t s) {
    switch (tn) {
        case 2: return launch_one<TM, 2>(g, splitk, s);
        case 3: return launch_one<TM, 3>(g, splitk, s);
        case 4: return launch_one<TM, 4>(g, splitk, s);
        case 5: return launch_one<TM, 5>(g, splitk, s);
        case 6: return launch_one<TM, 6>(g, splitk, s);
        case 7: return launch_one<TM, 7>(g, splitk, s);
        case 8: return launch_one<TM, 8>(g, splitk, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

// Environment override for tuning runs and tests: SDV2_GEMM_TILE="tm,tn,splitk" (read at every call).
static bool tile_override(TilePlan* p) {
    const char* e = getenv("SDV2_GEMM_TILE");
    int a, b, c;
    if (e && sscanf(e, "%d,%d,%d", &a, &b, &c) == 3 && a >= 1 && a <= 2 && b >= 2 && b <= 8 && c >= 1 && c <= 16) {
        *p = TilePlan{a, b, c};
        return true;
    }
    return false;
}

hipError_t launch_gemm_planned(const GemmArgs& g, int tm, int tn, int splitk, hipStream_t s) {
    if (g.epilogue == kEpiBias || g.epilogue == kEpiBiasGelu) splitk = 1;
    if (splitk > g.K / BK) splitk = 1;
    return tm == 1 ? launch_tn<1>(g, tn, splitk, s) : launch_tn<2>(g, tn, splitk, s);
}

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
    TilePlan p = plan_tiles(g.M, g.N, g.K, g.epilogue);
    tile_override(&p);
    return launch_gemm_planned(g, p.tm, p.tn, p.splitk, s);
}

}  // namespace sdv2
