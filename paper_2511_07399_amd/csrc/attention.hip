// Exact attention of a chunk's queries over a prefix of cache slots, flash style (online softmax,
// no score matrix in memory), for gfx950.
//
// This is the "4 b L_q L_kv C" term of the per-layer cost in Appendix B of the paper; the paper runs
// it with a FlashAttention kernel (Section 4.1) over the sink + rolling-window cache (Appendix D).
// Because resident tokens always occupy the slot prefix [0, kv_len) of the ring layout and softmax
// attention does not depend on the order of the keys, the kernel scans physical slots in order and
// needs no [sink | window] segment logic.  The same kernel serves the text cross-attention.
//
// Design
//   * Workgroup = 4 waves = 128 queries of one (stream, head); each wave owns 32 queries; two workgroups
//     per compute unit.
//   * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: keys are the rows,
//     queries the columns, so a lane (column = lane % 32) owns one query: its row maximum and row sum
//     live in that lane and its partner lane + 32, and the accumulator of S^T is already in the
//     register layout that the B operand of the second product O^T = V^T P^T wants.  No LDS round
//     trip for P.
//   * That needs V^T tiles with keys contiguous, which is why the cache stores values transposed
//     ([head][128][cap]); inside every group of 16 slots the cache swaps the middle two groups of four
//     (vt_column), which is the order in which the S^T accumulator holds its keys, so a V^T fragment is one
//     16-byte LDS read.  K tiles are contiguous 16 KB blocks of the [head][cap][128] key cache.
//   * K and V^T tiles of 64 keys go global -> LDS directly (global_load_lds_dwordx4), two stages each.  The
//     LDS swizzle is applied on the global side: K rows (256 B) XOR the 16-byte chunk index with row % 16,
//     V^T rows (128 B) with (row / 2) % 8, so that fragment reads are conflict free on the 64-bank LDS.
//   * The loop is software pipelined inside a wave: while the vector unit runs the softmax of tile t, the
//     matrix unit computes S^T of tile t + 1; the P V product of tile t follows.  The softmax costs about
//     as many vector cycles as the tile costs matrix cycles, so without this overlap (and that between
//     the two workgroups of a unit) the matrix unit idles half of the time.
//   * The exponents' reference point of a query trails its running maximum loosely instead of tracking it: the
//     steady-state loop forms no row maximum and rescales nothing; a sum of exponentials that leaves the range
//     sends the wave to a slow path that moves the reference point (it cancels in O / l).
//   * Skinny launches (few query tiles x heads) split the key range over several workgroups, which
//     write normalised partial outputs with their (max, sum); a small kernel merges them.
#include "common.h"

#include <stdio.h>
#include <stdlib.h>

#include <mutex>
#include <type_traits>

namespace sdv2 {

namespace {

constexpr int KT = 64;        // keys per tile
constexpr float kMaxSlack = 8.0f;   // log2 units within which a query's exponent reference is left where it is
constexpr float kNoKey = -1.0e30f;  // reference point of a query that has seen no key yet (key-split form)
constexpr float kSumLimit = 16384.0f;   // a lane's sum of p over one tile (at most 32 keys) beyond this: move the reference
constexpr int D = kHeadDim;
constexpr int K_TILE_BYTES = KT * D * 2;
constexpr int V_TILE_BYTES = D * KT * 2;

// max of three with one instruction and no NaN canonicalisation of the operands (scores are never NaN for
// valid slots; masked ones are -inf)
__device__ __forceinline__ float max3_f32(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

__device__ __forceinline__ float max2_f32(float a, float b) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
// max of x over the lane pair (l, l ^ 32): one swap of the two 32-lane halves on the vector unit (a shuffle
// through the LDS crossbar would put its latency on the path to the exponentials)
__device__ __forceinline__ float max_xor32(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return max2_f32(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Makes the compiler hold the fragments in registers at this point of the program (an empty statement that claims to
// read and write them): conversions to bf16 cannot be moved past it.
template <int N>
__device__ __forceinline__ void pin_fragments(bf16x8 (&f)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(f[i]));
}

typedef __attribute__((address_space(3))) void* lds_void_ptr;
__device__ __forceinline__ void load_to_lds_b128(const void* src, void* dst) {
    __builtin_amdgcn_global_load_lds(src, (lds_void_ptr)dst, 16, 0, 0);
}

template <int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attention_kernel(AttnArgs a, float scale_log2e) {
    constexpr int QT = 32 * NW;                   // queries per workgroup: one 32-query block per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    unsigned char* const k_stage = smem_raw;                          // [2][64 keys][256 B]
    unsigned char* const v_stage = smem_raw + 2 * K_TILE_BYTES;       // [2][128 d][128 B]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31;
    const int lh = lane >> 5;

    // Workgroups are handed to the eight XCDs in turn; renumber them so that each XCD (its own L2) works through
    // a contiguous run of (query tile, head, stream/split) triples, query tile fastest: the workgroups that
    // share a head's K and V then sit behind the same L2.
    const unsigned n_wg = gridDim.x * gridDim.y * gridDim.z;
    const unsigned flat = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const unsigned xcd = flat & 7u, per = n_wg >> 3, rem = n_wg & 7u;
    const unsigned logical = xcd * per + min(xcd, rem) + (flat >> 3);
    const int qt = (int)(logical % gridDim.x);
    const int h = (int)((logical / gridDim.x) % gridDim.y);
    const int bz = (int)(logical / (gridDim.x * gridDim.y));
    const int b = bz / a.splits;
    const int split = bz - b * a.splits;
    const int C = a.H * D;

    const int kv_len = __builtin_amdgcn_readfirstlane(a.desc ? a.desc->kv_len[b] : a.kv_len[b]);
    const int cap = a.cap[b];
    const int n_tiles = (kv_len + KT - 1) / KT;
    const int t0 = (int)((long long)split * n_tiles / a.splits);
    const int t1 = (int)((long long)(split + 1) * n_tiles / a.splits);
    const int tail_tile = (kv_len % KT) ? n_tiles - 1 : -1;           // the tile with slots past kv_len, if any

    // ---- this lane's query (column of S^T) and its eight d-step fragments
    const int q_in_chunk = qt * QT + wave * 32 + l31;
    const size_t q_row = (size_t)b * a.L + min(q_in_chunk, a.L - 1);
    bf16x8 qf[D / 16];
    {
        const bf16* qp = a.q + q_row * C + h * D + lh * 8;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + s * 16);
    }

    // ---- direct loads.  A wave load fills 1 KB of LDS in lane order: 4 K rows or 8 V^T rows.  Wave w issues
    // loads w, w + NW, ... of each tile; the XOR term of a lane's chunk is the same for all of them.
    const unsigned char* kbase = reinterpret_cast<const unsigned char*>(a.k[b] + (size_t)h * cap * D);
    const unsigned char* vbase = reinterpret_cast<const unsigned char*>(a.vt[b] + (size_t)h * D * cap);
    constexpr int LPT = 16 / NW;                  // wave loads per K tile and per V^T tile for each wave
    const int k_row = 4 * wave + (lane >> 4);                                     // + 4 NW i
    const uint32_t k_off = (uint32_t)k_row * 256u + (uint32_t)(((lane & 15) ^ (k_row & 15)) * 16);
    const int v_row = 8 * wave + (lane >> 3);                                     // + 8 NW i
    const size_t v_off = (size_t)v_row * cap * 2 + (size_t)(((lane & 7) ^ ((v_row >> 1) & 7)) * 16);
    auto load_k = [&](int t, int stage) {
        const unsigned char* src = kbase + (size_t)t * K_TILE_BYTES + k_off;
        unsigned char* dst = k_stage + stage * K_TILE_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < LPT; ++i) load_to_lds_b128(src + i * (NW * 1024), dst + i * (NW * 1024));
    };
    auto load_v = [&](int t, int stage) {
        const unsigned char* src = vbase + (size_t)t * (KT * 2) + v_off;
        unsigned char* dst = v_stage + stage * V_TILE_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < LPT; ++i) load_to_lds_b128(src + (size_t)i * (8 * NW) * cap * 2, dst + i * (NW * 1024));
    };
    // Slots past kv_len may hold anything (NaN included) and 0 x NaN is not 0: blank them in the staged V^T tile.
    auto blank_v_tail = [&](int t, int stage) {
        const int n_valid = kv_len - t * KT;
        bf16* sv = reinterpret_cast<bf16*>(v_stage + stage * V_TILE_BYTES);
        for (int idx = tid; idx < D * 8; idx += 64 * NW) {
            const int row = idx >> 3, p = idx & 7;
            const int c = p ^ ((row >> 1) & 7);
            bf16x8 v = *reinterpret_cast<bf16x8*>(sv + row * KT + p * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int u = 8 * c + e;                                          // stored column
                const int slot = (u & ~12) | ((u & 4) << 1) | ((u & 8) >> 1);     // slot it holds (vt_column is an involution)
                if (slot >= n_valid) v[e] = (bf16)0.0f;
            }
            *reinterpret_cast<bf16x8*>(sv + row * KT + p * 8) = v;
        }
    };

    f32x16 o_acc[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[i][r] = 0.0f;
    float m_run = -INFINITY;     // reference point of this query's exponents: within kMaxSlack below the running maximum of its scaled (log2-domain) scores
    float l_run = 0.0f;          // this lane's share of the running sum

    // Half of S^T of the tile in stage sk: d steps 4 half .. 4 half + 3 of both 32-key blocks.  The eight K
    // fragments are read first, the MFMAs alternate between the two accumulators (a dependent MFMA would
    // wait 12 clocks longer for its predecessor).
    auto qk_half = [&](f32x16 (&s)[2], const unsigned char* sk, int half, auto&& after_reads) {
        if (half == 0) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = 0.0f;
        }
        bf16x8 kf[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                kf[i][kb] = *reinterpret_cast<const bf16x8*>(sk + (kb * 32 + l31) * 256 +
                                                             (((2 * (4 * half + i) + lh) ^ (l31 & 15)) << 4));
        after_reads();
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i][kb], qf[4 * half + i], s[kb], 0, 0, 0);
    };
    auto nothing = []() {};

    auto wait_loads = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); };       // vmcnt(0) only
    auto barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    f32x16 s_a[2], s_b[2];
    // one tile: s_cur holds S^T of tile t; S^T of tile t + 1 is formed into s_nxt on the way
    // (tail: compile-time flag of the one tile that has slots past kv_len, so that the others carry no masking code)
    // (par: compile-time parity of t - t0, which picks the stages: their offsets are then immediates of the LDS reads)
    auto tile_step = [&](auto tail_c, auto par_c, f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2], int t) {
        constexpr bool tail = decltype(tail_c)::value;
        constexpr int rel = decltype(par_c)::value;
        wait_loads();
        barrier();                       // K(t+1) and V(t) have landed; everyone is done with K(t), V(t-1)
        if (tail) {
            blank_v_tail(t, rel & 1);
            __syncthreads();
        }
        const unsigned char* sk = k_stage + ((rel + 1) & 1) * K_TILE_BYTES;
        const unsigned char* sv = v_stage + (rel & 1) * V_TILE_BYTES;

        if (tail) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (t * KT + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3) >= kv_len) s_cur[kb][r] = -INFINITY;
        }
        // ---- S^T(t+1) on the matrix unit in two halves | under each, p = 2^(s c - m_run) of one 32-key block of
        // tile t on the vector unit, its row sum and its bf16 fragments.  m_run is the exponents' reference point, not
        // the exact running maximum: no maximum is formed here at all.  If a score has run more than about
        // log2(kSumLimit) ahead of it (or no key has been seen yet: m_run = -inf makes p infinite), this lane's sum of
        // p leaves the range, and the wave then takes the slow path below, which moves the reference point to the
        // true maximum, rescales the accumulators and forms p again.  The reference cancels in O / l.
        // (Past the last tile the matrix unit reads a stale stage and the result is dropped: no branch, so that matrix
        // and vector instructions share a basic block and can be interleaved.)
        // The loads of K(t+2) and V(t+1) go out between the first MFMAs, one each: issued in a burst after the barrier they
        // hold every wave of the unit (an issuing wave waits while the LDS pipeline takes in the loads before its own,
        // about 25 clocks each) with the matrix pipe idle.  They are unconditional: past the last tile they fetch it
        // again into a stage that nobody reads, so that matrix, vector and load instructions share a basic block.
        float ls[4];
        bf16x8 pf[4];
        auto exps = [&](int kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[kb][r], scale_log2e, -m_run));
                ls[r & 3] = (kb == 0 && r < 4) ? p : ls[r & 3] + p;     // four independent chains
                pf[kb * 2 + (r >> 3)][r & 7] = (bf16)p;
            }
        };
        __builtin_amdgcn_sched_barrier(0);
        qk_half(s_nxt, sk, 0, [&]() {
            load_k(min(t + 2, t1 - 1), rel & 1);
            load_v(min(t + 1, t1 - 1), (rel + 1) & 1);
        });
        exps(0);
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);       // the eight fragment reads, then MFMA | load | vector work
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (m < 2 * LPT) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        qk_half(s_nxt, sk, 1, nothing);
        exps(1);
        float lsum = (ls[0] + ls[1]) + (ls[2] + ls[3]);
        pin_fragments(pf);               // the bf16 fragments are formed here, among the MFMAs, not after the branch
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(lsum <= kSumLimit)) != 0, 0)) {
            // Slow path: move the reference point to the true row maximum (four independent chains; the same for the
            // two lanes of a query), rescale the accumulators and form p again.
            float mc[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                mc[c] = max3_f32(s_cur[0][4 * c], s_cur[1][4 * c], s_cur[0][4 * c + 1]);
                mc[c] = max3_f32(mc[c], s_cur[1][4 * c + 1], s_cur[0][4 * c + 2]);
                mc[c] = max3_f32(mc[c], s_cur[1][4 * c + 2], s_cur[0][4 * c + 3]);
                mc[c] = max2_f32(mc[c], s_cur[1][4 * c + 3]);
            }
            const float mx = max_xor32(max2_f32(max3_f32(mc[0], mc[1], mc[2]), mc[3]));
            const float m_new = fmaxf(m_run, mx * scale_log2e);     // finite: every tile has a valid key
            const bool moved = m_new > m_run + kMaxSlack;            // a query within kMaxSlack of its reference keeps it
            const float alpha = moved ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.0f;
            l_run *= alpha;
#pragma unroll
            for (int i = 0; i < D / 32; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[i][r] *= alpha;
            m_run = moved ? m_new : m_run;
            exps(0);
            exps(1);
            lsum = (ls[0] + ls[1]) + (ls[2] + ls[3]);
            pin_fragments(pf);
        }
        l_run += lsum;
        __builtin_amdgcn_sched_barrier(0);

        // ---- O^T += V^T P^T : four steps of 16 keys; step ts uses registers 8 (ts % 2) .. + 7 of block ts / 2,
        // i.e. slots 16 ts + 4 (lane / 32) + {0..3} and 16 ts + 8 + 4 (lane / 32) + {0..3}: chunk 2 ts + lane / 32
        // of the V^T row in the cache's column order.
#pragma unroll
        for (int ts = 0; ts < 4; ++ts) {
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const unsigned char* vrow = sv + (db * 32 + l31) * 128;
                const bf16x8 vf = *reinterpret_cast<const bf16x8*>(vrow + (((2 * ts + lh) ^ ((l31 >> 1) & 7)) << 4));
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ts], o_acc[db], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);       // fragment reads run six ahead of the MFMAs
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    if (t0 < t1) {
        load_k(t0, 0);
        load_v(t0, 0);
        if (t0 + 1 < t1) load_k(t0 + 1, 1);
        wait_loads();
        barrier();
        qk_half(s_a, k_stage, 0, nothing);
        qk_half(s_a, k_stage, 1, nothing);
    }
    // full tiles in pairs (the two S^T register sets trade places), then what is left: at most one full tile
    // and the tail tile
    const int t_full = (t1 - 1 == tail_tile) ? t1 - 1 : t1;          // tiles [t0, t_full) have 64 valid slots
    const std::false_type no_tail;
    const std::true_type with_tail;
    const std::integral_constant<int, 0> even;
    const std::integral_constant<int, 1> odd;
    int t = t0;
    for (; t + 2 <= t_full; t += 2) {
        tile_step(no_tail, even, s_a, s_b, t);
        tile_step(no_tail, odd, s_b, s_a, t + 1);
    }
    if (t < t_full) {
        tile_step(no_tail, even, s_a, s_b, t);
        if (t_full < t1) tile_step(with_tail, odd, s_b, s_a, t_full);
    } else if (t_full < t1) {
        tile_step(with_tail, even, s_a, s_b, t_full);
    }

    // ---- finish: divide by the row sum and write
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    const float inv_l = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    if (q_in_chunk >= a.L) return;
    if (a.splits == 1) {
        bf16* op = a.o + q_row * C + h * D + 4 * lh;
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (bf16)(o_acc[db][4 * g + e] * inv_l);
                *reinterpret_cast<bf16x4*>(op + db * 32 + 8 * g) = w;
            }
        }
    } else {
        const size_t rows = (size_t)a.B * a.L;
        float* op = a.part_o + ((size_t)split * rows + q_row) * C + h * D + 4 * lh;
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = o_acc[db][4 * g + e] * inv_l;
                *reinterpret_cast<f32x4*>(op + db * 32 + 8 * g) = w;
            }
        }
        if (lh == 0) {
            float* ml = a.part_ml + (((size_t)split * rows + q_row) * a.H + h) * 2;
            ml[0] = m_run;
            ml[1] = l_tot;
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Key-split form for skinny launches (a single 1024-token chunk: heads x query tiles is well below the number of
// SIMDs).  A workgroup is NQ query blocks x NKW key slices = 8 waves: it walks the whole key range in tiles of
// 32 NKW keys, wave (qb, kw) computing the scores of its 32 queries against keys 32 kw .. 32 kw + 31 of every tile
// and keeping its own running maximum, sum and output; at the end the NKW partial results of a query block are
// merged through LDS.  Compared with splitting the key range over workgroups this needs no partial outputs in
// memory and no merge kernel, and every K / V^T tile staged in LDS still serves all eight waves.
//   K stage:   32 NKW keys x 256 B, chunk c of row r at position c ^ (r % 16)
//   V^T stage: 128 rows (d) x 32 NKW keys (64 NKW bytes; 256 B for NKW = 4), same swizzle
// Needs cap % (32 NKW) == 0 (a tile never reaches past a V^T row).
template <int NQ, int NKW>
__global__ __launch_bounds__(64 * NQ * NKW, 1) void attention_ks_kernel(AttnArgs a, float scale_log2e) {
    static_assert(NKW == 4 && NQ * NKW == 8, "tiles of 128 keys, eight waves");
    constexpr int NW = NQ * NKW;
    constexpr int QT = 32 * NQ;
    constexpr int KTT = 32 * NKW;                         // keys per tile
    constexpr int ROWB = 256;                             // bytes per LDS row of either stage
    constexpr int K_BYTES = KTT * ROWB;                   // 32 KB
    constexpr int V_BYTES = D * ROWB;                     // 32 KB
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    unsigned char* const k_stage = smem_raw;                          // [2][K_BYTES]
    unsigned char* const v_stage = smem_raw + 2 * K_BYTES;            // [2][V_BYTES]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qb = wave % NQ;
    const int kw = wave / NQ;
    const int l31 = lane & 31;
    const int lh = lane >> 5;

    const unsigned n_wg = gridDim.x * gridDim.y * gridDim.z;
    const unsigned flat = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const unsigned xcd = flat & 7u, per = n_wg >> 3, rem = n_wg & 7u;
    const unsigned logical = xcd * per + min(xcd, rem) + (flat >> 3);
    const int qt = (int)(logical % gridDim.x);
    const int h = (int)((logical / gridDim.x) % gridDim.y);
    const int b = (int)(logical / (gridDim.x * gridDim.y));
    const int C = a.H * D;

    const int kv_len = __builtin_amdgcn_readfirstlane(a.desc ? a.desc->kv_len[b] : a.kv_len[b]);
    const int cap = a.cap[b];
    const int n_tiles = (kv_len + KTT - 1) / KTT;
    const int tail_tile = (kv_len % KTT) ? n_tiles - 1 : -1;

    const int q_in_chunk = qt * QT + qb * 32 + l31;
    const size_t q_row = (size_t)b * a.L + min(q_in_chunk, a.L - 1);
    bf16x8 qf[D / 16];
    {
        const bf16* qp = a.q + q_row * C + h * D + lh * 8;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + s * 16);
    }

    // A wave load fills four 256-byte rows; wave w issues loads w, w + 8, w + 16, w + 24 of each tile.
    const unsigned char* kbase = reinterpret_cast<const unsigned char*>(a.k[b] + (size_t)h * cap * D);
    const unsigned char* vbase = reinterpret_cast<const unsigned char*>(a.vt[b] + (size_t)h * D * cap);
    constexpr int LPT = KTT / 4 / NW;                     // 4 wave loads per tile and operand for each wave
    const int ld_row = 4 * wave + (lane >> 4);                                    // + 32 i
    const int ld_chunk = (lane & 15) ^ (ld_row & 15);                             // 32 i does not change row % 16
    const uint32_t k_off = (uint32_t)ld_row * ROWB + (uint32_t)ld_chunk * 16;
    const size_t v_off = (size_t)ld_row * cap * 2 + (size_t)ld_chunk * 16;
    // (a tile index past the last tile fetches the last tile again, into a stage that nobody reads any more: the loads
    // are unconditional so that they can sit among the matrix instructions of a basic block)
    auto load_k = [&](int t, int stage) {
        const unsigned char* src = kbase + (size_t)min(t, n_tiles - 1) * K_BYTES + k_off;
        unsigned char* dst = k_stage + stage * K_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < LPT; ++i) load_to_lds_b128(src + i * (NW * 1024), dst + i * (NW * 1024));
    };
    auto load_v = [&](int t, int stage) {
        const unsigned char* src = vbase + (size_t)min(t, n_tiles - 1) * (KTT * 2) + v_off;
        unsigned char* dst = v_stage + stage * V_BYTES + wave * 1024;
#pragma unroll
        for (int i = 0; i < LPT; ++i) load_to_lds_b128(src + (size_t)i * 32 * cap * 2, dst + i * (NW * 1024));
    };
    // Slots past kv_len may hold anything (NaN included) and 0 x NaN is not 0: blank them in the staged V^T tile.
    auto blank_v_tail = [&](int t, int stage) {
        const int n_valid = kv_len - t * KTT;
        bf16* sv = reinterpret_cast<bf16*>(v_stage + stage * V_BYTES);
        for (int idx = tid; idx < D * 16; idx += 64 * NW) {
            const int row = idx >> 4, p = idx & 15;
            const int c = p ^ (row & 15);
            bf16x8 v = *reinterpret_cast<bf16x8*>(sv + row * (ROWB / 2) + p * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int u = 8 * c + e;                                          // stored column
                const int slot = (u & ~12) | ((u & 4) << 1) | ((u & 8) >> 1);     // slot it holds
                if (slot >= n_valid) v[e] = (bf16)0.0f;
            }
            *reinterpret_cast<bf16x8*>(sv + row * (ROWB / 2) + p * 8) = v;
        }
    };

    f32x16 o_acc[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[i][r] = 0.0f;
    float m_run = kNoKey;        // finite: a fully masked slice has scores of -inf, and -inf + inf is not a number
    float l_run = 0.0f;

    // Half of S^T of this wave's 32 keys of the tile in stage sk: d steps 4 half .. 4 half + 3.
    // this lane's eight K fragments and its two V^T fragments of a step in the first 32-row block, all in stage 0: the
    // stage and the block add compile-time constants, which the LDS reads take as immediates
    const unsigned char* kfrag[D / 16];
#pragma unroll
    for (int i = 0; i < D / 16; ++i) kfrag[i] = k_stage + (kw * 32 + l31) * ROWB + (((2 * i + lh) ^ (l31 & 15)) << 4);
    const unsigned char* vfrag[2];
#pragma unroll
    for (int ts = 0; ts < 2; ++ts) vfrag[ts] = v_stage + l31 * ROWB + (((4 * kw + 2 * ts + lh) ^ (l31 & 15)) << 4);
    auto qk_half = [&](f32x16& s, int stage, int half, auto&& after_reads) {
        if (half == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.0f;
        }
        bf16x8 kf[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            kf[i] = *reinterpret_cast<const bf16x8*>(kfrag[4 * half + i] + stage * K_BYTES);
        after_reads();
#pragma unroll
        for (int i = 0; i < 4; ++i) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[4 * half + i], s, 0, 0, 0);
    };
    auto nothing = []() {};
    auto wait_loads = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); };       // vmcnt(0) only
    auto barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    f32x16 s_a, s_b;
    auto tile_step = [&](auto tail_c, auto par_c, f32x16& s_cur, f32x16& s_nxt, int t) {
        constexpr bool tail = decltype(tail_c)::value;
        constexpr int par = decltype(par_c)::value;      // parity of t, at compile time: stage offsets become immediates
        wait_loads();
        barrier();                       // K(t+1) and V(t) have landed; everyone is done with K(t), V(t-1)
        if (tail) {
            blank_v_tail(t, par);
            __syncthreads();
        }
        constexpr int sk = par ^ 1;          // stage of K(t+1)
        if (tail) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (t * KTT + kw * 32 + 8 * (r >> 2) + 4 * lh + (r & 3) >= kv_len) s_cur[r] = -INFINITY;
        }
        // ---- S^T(t+1) on the matrix unit in two halves | p of tile t on the vector unit, without a row maximum
        // (see attention_kernel): the slow path is taken when a sum of p has left the range, which is also what
        // happens at a lane's first valid key (m_run = kNoKey: p infinite).  A lane whose slice lies past kv_len has
        // scores of -inf, p = 0 and keeps kNoKey (finite, so that -inf - m_run is not "not a number").
        float ls[4];
        bf16x8 pf[2];
        auto exps = [&](int h) {
#pragma unroll
            for (int r = 8 * h; r < 8 * h + 8; ++r) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[r], scale_log2e, -m_run));
                ls[r & 3] = r < 4 ? p : ls[r & 3] + p;
                pf[r >> 3][r & 7] = (bf16)p;
            }
        };
        __builtin_amdgcn_sched_barrier(0);
        // the loads of K(t+2) go out between the MFMAs of the first half, those of V(t+1) between those of the second
        qk_half(s_nxt, sk, 0, [&]() { load_k(t + 2, par); });
        exps(0);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        qk_half(s_nxt, sk, 1, [&]() { load_v(t + 1, par ^ 1); });
        exps(1);
        float lsum = (ls[0] + ls[1]) + (ls[2] + ls[3]);
        pin_fragments(pf);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(lsum <= kSumLimit)) != 0, 0)) {
            float mc[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) mc[c] = max2_f32(max3_f32(s_cur[4 * c], s_cur[4 * c + 1], s_cur[4 * c + 2]), s_cur[4 * c + 3]);
            const float mx = max_xor32(max2_f32(max3_f32(mc[0], mc[1], mc[2]), mc[3]));
            const float m_new = fmaxf(m_run, mx * scale_log2e);       // stays kNoKey in a lane that has still seen no key
            const bool moved = m_new > m_run + kMaxSlack;
            const float al = moved ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.0f;
            l_run *= al;
#pragma unroll
            for (int i = 0; i < D / 32; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[i][r] *= al;
            m_run = moved ? m_new : m_run;
            exps(0);
            exps(1);
            lsum = (ls[0] + ls[1]) + (ls[2] + ls[3]);
            pin_fragments(pf);
        }
        l_run += lsum;
        __builtin_amdgcn_sched_barrier(0);
        // ---- O^T += V^T P^T: two steps of 16 keys; chunk 4 kw + 2 ts + lh of the V^T row in the cache's column order
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) {
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const bf16x8 vf = *reinterpret_cast<const bf16x8*>(vfrag[ts] + par * V_BYTES + db * 32 * ROWB);
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ts], o_acc[db], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    load_k(0, 0);
    load_v(0, 0);
    if (1 < n_tiles) load_k(1, 1);
    wait_loads();
    barrier();
    qk_half(s_a, 0, 0, nothing);
    qk_half(s_a, 0, 1, nothing);
    const int t_full = (tail_tile >= 0) ? n_tiles - 1 : n_tiles;        // tiles [0, t_full) have 128 valid slots
    const std::false_type no_tail;
    const std::true_type with_tail;
    const std::integral_constant<int, 0> even;
    const std::integral_constant<int, 1> odd;
    int t = 0;
    for (; t + 2 <= t_full; t += 2) {
        tile_step(no_tail, even, s_a, s_b, t);
        tile_step(no_tail, odd, s_b, s_a, t + 1);
    }
    if (t < t_full) {
        tile_step(no_tail, even, s_a, s_b, t);
        if (t_full < n_tiles) tile_step(with_tail, odd, s_b, s_a, t_full);
    } else if (t_full < n_tiles) {
        tile_step(with_tail, even, s_a, s_b, t_full);
    }

    // ---- merge the NKW partial results of each query block through LDS (the stages are free now)
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    float* const xm = reinterpret_cast<float*>(smem_raw + 4 * K_BYTES);           // [NW][32] maxima, after the stages
    float* const xl = xm + NW * 32;                                               // [NW][32] sums
    float* const ox = reinterpret_cast<float*>(smem_raw);                         // [NW][4][16][64] weighted outputs
    __syncthreads();
    if (lh == 0) {
        xm[wave * 32 + l31] = m_run;
        xl[wave * 32 + l31] = l_tot;
    }
    __syncthreads();
    // a slice that saw no key has m = kNoKey and l = 0: weight 2^(kNoKey - mmax) = 0, or 1 times l = 0 if all are such
    float mmax = kNoKey;
#pragma unroll
    for (int k = 0; k < NKW; ++k) mmax = fmaxf(mmax, xm[(qb + NQ * k) * 32 + l31]);
    float lsum = 0.0f;
#pragma unroll
    for (int k = 0; k < NKW; ++k)
        lsum += xl[(qb + NQ * k) * 32 + l31] * __builtin_amdgcn_exp2f(xm[(qb + NQ * k) * 32 + l31] - mmax);
    const float wgt = lsum > 0.0f ? __builtin_amdgcn_exp2f(m_run - mmax) / lsum : 0.0f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) ox[((wave * 4 + db) * 16 + r) * 64 + lane] = o_acc[db][r] * wgt;
    __syncthreads();
    if (q_in_chunk >= a.L) return;
    // wave (qb, kw) adds up and writes the 32 channels db = kw of its query block
    bf16* op = a.o + q_row * C + h * D + kw * 32 + 4 * lh;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float acc = 0.0f;
#pragma unroll
            for (int k = 0; k < NKW; ++k) acc += ox[(((qb + NQ * k) * 4 + kw) * 16 + 4 * g + e) * 64 + lane];
            w[e] = (bf16)acc;
        }
        *reinterpret_cast<bf16x4*>(op + 8 * g) = w;
    }
}

// out = sum_i w_i O_i / sum_i w_i,  w_i = l_i 2^(m_i - max m).  One thread per four channels.
__global__ __launch_bounds__(256) void attention_merge_kernel(AttnArgs a) {
    const int C = a.H * D;
    const size_t rows = (size_t)a.B * a.L;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;     // over rows * C / 4
    if (idx >= rows * (C / 4)) return;
    const size_t row = idx / (C / 4);
    const int c4 = (int)(idx - row * (C / 4)) * 4;
    const int h = c4 / D;
    float m[16], l[16];
    float mmax = -INFINITY;
    for (int s = 0; s < a.splits; ++s) {
        const float* ml = a.part_ml + (((size_t)s * rows + row) * a.H + h) * 2;
        m[s] = ml[0];
        l[s] = ml[1];
        mmax = fmaxf(mmax, m[s]);
    }
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    float wsum = 0.0f;
    for (int s = 0; s < a.splits; ++s) {
        const float w = l[s] > 0.0f ? l[s] * __builtin_amdgcn_exp2f(m[s] - mmax) : 0.0f;
        const f32x4 o = *reinterpret_cast<const f32x4*>(a.part_o + ((size_t)s * rows + row) * C + c4);
        acc += o * w;
        wsum += w;
    }
    const float inv = 1.0f / wsum;
    bf16x4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = (bf16)(acc[e] * inv);
    *reinterpret_cast<bf16x4*>(a.o + row * C + c4) = out;
}

}  // namespace

// Waves per workgroup: 4 (128 queries, two workgroups per compute unit) or 8 (256 queries, one workgroup per unit,
// half the K/V traffic from the L2 per query).
// Overrides for tuning runs and tests, set through sdv2_tuning_set("attn_waves" / "attn_splits", ...); 0 = the plan's
// own choice.  attn_waves 4 / 8: that many query blocks per workgroup, one key stream; 2: the key-split form.
static int g_force_waves = 0;
static int g_force_splits = 0;
void set_attention_overrides(int waves, int splits) {
    if (waves >= 0) g_force_waves = (waves == 4 || waves == 8 || waves == 2) ? waves : 0;
    if (splits >= 0) g_force_splits = splits > 16 ? 16 : splits;
}

// Key-split form (2 query blocks x 4 key slices): when 128-query workgroups would give fewer than three quarters of
// the compute units a workgroup each, and every stream's capacity is a whole number of its 128-key tiles.
static bool attention_plan_key_split(const AttnArgs& a) {
    for (int b = 0; b < a.B; ++b)
        if (a.cap[b] % 128) return false;
    if (g_force_waves) return g_force_waves == 2;
    return ((a.L + 127) / 128) * a.H * a.B < 192;
}

// Waves per workgroup: 4 (128 queries, two workgroups per compute unit) or 8 (256 queries, one workgroup per unit,
// half the K/V traffic from the L2 per query).
int attention_plan_waves(int B, int L, int H, int max_kv_len) {
    if (g_force_waves == 4 || g_force_waves == 8) return g_force_waves;
    (void)max_kv_len;
    // 256-query workgroups only where they still give at least half of the compute units a workgroup each
    return ((L + 255) / 256) * H * B >= 128 ? 8 : 4;
}

int attention_plan_splits(int B, int L, int H, int max_kv_len) {
    const int forced = g_force_splits;
    const int QT = 32 * attention_plan_waves(B, L, H, max_kv_len);
    const int slots = QT == 128 ? 512 : 256;         // workgroups resident at once
    const int n_tiles = (max_kv_len + KT - 1) / KT;
    int splits = 1;
    if (forced > 0) {
        splits = forced;
    } else {
        // Two workgroups fit a compute unit: aim at no more than 512 workgroups in all, keep at least six
        // key tiles per split (the merge pass costs about as much as two tiles), and do not split at all
        // once every unit has a workgroup.
        const int wgs = ((L + QT - 1) / QT) * H * B;
        if (wgs < slots / 2) {
            splits = slots / wgs;
            while (splits > 1 && n_tiles / splits < 6) --splits;
        }
    }
    while (splits > 1 && n_tiles / splits < 2) --splits;
    return splits > 16 ? 16 : splits;
}

size_t attention_workspace_bytes(int B, int L, int C, int max_kv_len) {
    const int H = C / D;
    const int splits = attention_plan_splits(B, L, H, max_kv_len);
    if (splits == 1) return 0;
    const size_t rows = (size_t)B * L;
    return (size_t)splits * rows * C * sizeof(float) + (size_t)splits * rows * H * 2 * sizeof(float);
}

void attention_plan_name(const AttnArgs& a, char* out, size_t cap) {
    int max_kv = 0;
    for (int b = 0; b < a.B; ++b) max_kv = a.kv_len[b] > max_kv ? a.kv_len[b] : max_kv;
    if (attention_plan_key_split(a)) snprintf(out, cap, "attention_ks_kernel<2, 4>");
    else snprintf(out, cap, "attention_kernel<%d>", attention_plan_waves(a.B, a.L, a.H, max_kv));
}

bool attention_has_merge_pass(const AttnArgs& a) { return a.splits > 1 && !attention_plan_key_split(a); }

hipError_t launch_attention(const AttnArgs& a, hipStream_t s, int part) {
    const size_t smem = (size_t)2 * K_TILE_BYTES + 2 * V_TILE_BYTES;
    constexpr size_t smem_ks = (size_t)4 * 32768 + 2 * 8 * 32 * sizeof(float);     // four 32 KB stages + the (m, l) exchange
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&]() {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel<4>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (attr_err == hipSuccess)
            attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel<8>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (attr_err == hipSuccess)
            attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_ks_kernel<2, 4>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_ks);
    });
    if (attr_err != hipSuccess || attributes_only()) return attr_err;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
    if (attention_plan_key_split(a)) {
        if (part == 2) return hipSuccess;
        dim3 grid((a.L + 63) / 64, a.H, a.B);
        hipLaunchKernelGGL((attention_ks_kernel<2, 4>), grid, dim3(512), smem_ks, s, a, scale_log2e);
        return hipGetLastError();
    }
    hipError_t e = hipSuccess;
    if (part != 2) {
        int max_kv = 0;
        for (int b = 0; b < a.B; ++b) max_kv = a.kv_len[b] > max_kv ? a.kv_len[b] : max_kv;
        const int nw = attention_plan_waves(a.B, a.L, a.H, max_kv);
        const int QT = 32 * nw;
        dim3 grid((a.L + QT - 1) / QT, a.H, a.B * a.splits);
        if (nw == 8) hipLaunchKernelGGL(attention_kernel<8>, grid, dim3(512), smem, s, a, scale_log2e);
        else hipLaunchKernelGGL(attention_kernel<4>, grid, dim3(256), smem, s, a, scale_log2e);
        e = hipGetLastError();
    }
    if (e != hipSuccess || part == 1) return e;
    if (a.splits > 1) {
        const size_t n = (size_t)a.B * a.L * (a.H * D / 4);
        hipLaunchKernelGGL(attention_merge_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace sdv2
