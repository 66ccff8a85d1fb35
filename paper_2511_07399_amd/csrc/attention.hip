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
//   * Workgroup = 4 waves = 128 queries of one (stream, head); each wave owns 32 queries.
//   * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: keys are the rows,
//     queries the columns, so a lane (column = lane % 32) owns one query: its row maximum and row sum
//     live in that lane and its partner lane + 32, and the accumulator of S^T is already in the
//     register layout that the B operand of the second product O^T = V^T P^T wants.  No LDS round
//     trip for P.
//   * That needs V^T tiles with keys contiguous, which is why the cache stores values transposed
//     ([head][128][cap]); K tiles are contiguous 16 KB blocks of the [head][cap][128] key cache.
//   * K and V^T tiles of 64 keys go global -> registers -> LDS, double buffered.  Rows are swizzled for
//     the 64-bank LDS: K rows (256 B) XOR the 16-byte chunk index with row % 16; V^T rows (128 B) XOR it
//     with (row / 2) % 8 and swap the two 8-byte halves of a chunk in rows 16..31 of each block of 32, so
//     that the 32 lanes of an 8-byte fragment read hit 32 different bank groups.
//   * Skinny launches (few query tiles x heads) split the key range over several workgroups, which
//     write normalised partial outputs with their (max, sum); a small kernel merges them.
#include "common.h"

#include <stdlib.h>

namespace sdv2 {

namespace {

constexpr int QT = 128;       // queries per workgroup
constexpr int KT = 64;        // keys per tile
constexpr int D = kHeadDim;
constexpr int STAGE = KT * D + D * KT;   // elements per LDS stage: K tile then V^T tile

__global__ __launch_bounds__(256, 2) void attention_kernel(AttnArgs a, float scale_log2e) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* const sm = reinterpret_cast<bf16*>(smem_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l31 = lane & 31;
    const int lh = lane >> 5;

    const int qt = blockIdx.x;
    const int h = blockIdx.y;
    const int b = blockIdx.z / a.splits;
    const int split = blockIdx.z - b * a.splits;
    const int C = a.H * D;

    const int kv_len = a.kv_len[b];
    const int cap = a.cap[b];
    const int n_tiles = (kv_len + KT - 1) / KT;
    const int t0 = (int)((long long)split * n_tiles / a.splits);
    const int t1 = (int)((long long)(split + 1) * n_tiles / a.splits);

    // ---- this lane's query (column of S^T) and its eight d-step fragments
    const int q_in_chunk = qt * QT + wave * 32 + l31;
    const size_t q_row = (size_t)b * a.L + min(q_in_chunk, a.L - 1);
    bf16x8 qf[D / 16];
    {
        const bf16* qp = a.q + q_row * C + h * D + lh * 8;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + s * 16);
    }

    // ---- global -> register staging of one K tile and one V^T tile
    const bf16* kbase = a.k[b] + (size_t)h * cap * D;
    const bf16* vbase = a.vt[b] + (size_t)h * D * cap;
    bf16x8 rk[4], rv[4];
    auto gload = [&](int t) {
        const bf16* kp = kbase + (size_t)t * KT * D;
#pragma unroll
        for (int i = 0; i < 4; ++i) rk[i] = *reinterpret_cast<const bf16x8*>(kp + (tid + 256 * i) * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx >> 3, c = idx & 7;
            rv[i] = *reinterpret_cast<const bf16x8*>(vbase + (size_t)row * cap + t * KT + c * 8);
            const int key0 = t * KT + c * 8;
            if (key0 + 8 > kv_len) {      // only in the last tile: slots past kv_len may hold anything
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (key0 + e >= kv_len) rv[i][e] = (bf16)0.0f;
            }
        }
    };
    auto sstore = [&](int buf) {
        bf16* sk = sm + buf * STAGE;
        bf16* sv = sk + KT * D;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx >> 4, c = idx & 15;
            *reinterpret_cast<bf16x8*>(sk + row * D + ((c ^ (row & 15)) << 3)) = rk[i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx >> 3, c = idx & 7;
            bf16x8 w = rv[i];
            if (row & 16) w = __builtin_shufflevector(w, w, 4, 5, 6, 7, 0, 1, 2, 3);
            *reinterpret_cast<bf16x8*>(sv + row * KT + ((c ^ ((row >> 1) & 7)) << 3)) = w;
        }
    };

    f32x16 o_acc[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[i][r] = 0.0f;
    float m_run = -INFINITY;     // running maximum of the scaled (log2-domain) scores of this query
    float l_run = 0.0f;          // this lane's share of the running sum

    // Loads and LDS writes of the next tile are unconditional (the tile index is clamped; the last
    // iteration re-stages its own tile into the idle buffer) so that the loop body is straight-line code
    // whose issue order can be laid out explicitly: global loads between the QK^T MFMAs, LDS writes
    // between the PV MFMAs, fragment reads one step ahead of the MFMAs that use them.
    if (t0 < t1) {
        gload(t0);
        sstore(0);
    }
    __syncthreads();
    for (int t = t0; t < t1; ++t) {
        const int buf = (t - t0) & 1;
        const bf16* sk = sm + buf * STAGE;
        const bf16* sv = sk + KT * D;
        __builtin_amdgcn_sched_barrier(0);
        gload(min(t + 1, t1 - 1));

        // ---- S^T = K Q^T for the tile's two blocks of 32 keys
        f32x16 s_acc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s_acc[kb][r] = 0.0f;
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sk + (kb * 32 + l31) * D +
                                                                    (((2 * s + lh) ^ (l31 & 15)) << 3));
                s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s_acc[kb], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (m & 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- online softmax in the log2 domain: p = 2^(s c - m), m = running maximum of s c
        const bool tail = (t + 1) * KT > kv_len;
        if (tail) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (t * KT + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3) >= kv_len) s_acc[kb][r] = -INFINITY;
        }
        float mx = fmaxf(s_acc[0][0], s_acc[1][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s_acc[0][r], s_acc[1][r]));
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float m_new = fmaxf(m_run, mx * scale_log2e);     // finite: every tile has a valid key
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {  // rescale only when some row's maximum moved
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            l_run *= alpha;
#pragma unroll
            for (int i = 0; i < D / 32; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[i][r] *= alpha;
            m_run = m_new;
        }
        float lsum = 0.0f;
        bf16x8 pf[4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][r], scale_log2e, -m_run));
                lsum += p;
                pf[kb * 2 + (r >> 3)][r & 7] = (bf16)p;
            }
        }
        l_run += lsum;
        __builtin_amdgcn_sched_barrier(0);

        // ---- O^T += V^T P^T : four steps of 16 keys; step ts uses registers 8 (ts % 2) .. +7 of block ts / 2,
        // i.e. keys 16 ts + 4 (lane / 32) + {0..3} and 16 ts + 8 + 4 (lane / 32) + {0..3}.
#pragma unroll
        for (int ts = 0; ts < 4; ++ts) {
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const bf16* vrow = sv + (db * 32 + l31) * KT + 4 * (lh ^ (l31 >> 4));
                const bf16x4 v0 = *reinterpret_cast<const bf16x4*>(vrow + (((2 * ts) ^ ((l31 >> 1) & 7)) << 3));
                const bf16x4 v1 = *reinterpret_cast<const bf16x4*>(vrow + (((2 * ts + 1) ^ ((l31 >> 1) & 7)) << 3));
                const bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ts], o_acc[db], 0, 0, 0);
            }
        }
        sstore(buf ^ 1);
        __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            if (m & 1) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
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

int attention_plan_splits(int B, int L, int H, int max_kv_len) {
    const char* e = getenv("SDV2_ATTN_SPLITS");      // tuning runs and tests; read at every call
    const int forced = e ? atoi(e) : 0;
    const int n_tiles = (max_kv_len + KT - 1) / KT;
    int splits = 1;
    if (forced > 0) {
        splits = forced;
    } else {
        // Two workgroups fit a compute unit: aim at no more than 512 workgroups in all, keep at least six
        // key tiles per split (the merge pass costs about as much as two tiles), and do not split at all
        // once every unit has a workgroup.
        const int wgs = ((L + QT - 1) / QT) * H * B;
        if (wgs < 256) {
            splits = 512 / wgs;
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

hipError_t launch_attention(const AttnArgs& a, hipStream_t s) {
    const size_t smem = (size_t)2 * STAGE * sizeof(bf16);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
    dim3 grid((a.L + QT - 1) / QT, a.H, a.B * a.splits);
    hipLaunchKernelGGL(attention_kernel, grid, dim3(256), smem, s, a, scale_log2e);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.splits > 1) {
        const size_t n = (size_t)a.B * a.L * (a.H * D / 4);
        hipLaunchKernelGGL(attention_merge_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace sdv2
