// Projections of a wide pass (9..16 sequences, bf16 weights) as a dense contraction on the matrix
// cores: v_mfma_f32_16x16x32_bf16 multiplies a tile of 16 weight rows x 32 columns by the staged
// inputs of 16 sequences over the same 32 columns.
//
// The paper keeps its row-partitioned matrix-vector scheme up to batch 4 (Section 5.2, larger batch
// sizes) and leaves more sequences open; at 16 sequences the 4x4x4 blocks of gemv_run_quad re-read
// every staged input once per group of four rows (eight LDS bytes per weight byte) and the
// projections become LDS- and issue-bound.  Here
//   * a WORKGROUP owns a contiguous range of rows (N / workgroups, in groups of four), cut into
//     tiles of 16; its four waves split K: within every staged K segment (2048 columns) wave w
//     multiplies columns [512 w, 512 w + 512) of ALL the workgroup's tiles, so each staged input
//     element is read from LDS once per tile by one wave only (two LDS bytes per weight byte);
//   * lane (r = lane % 16, g = lane / 16) loads 16 bytes of row r of the tile: per wave load 16 rows
//     x 64 contiguous bytes, eight of them (one ring stage) = 512 contiguous bytes per row, two
//     stages per (tile, segment); the same two-stage register ring as the other paths, refilled
//     across tile and segment boundaries;
//   * the 16x16 accumulators (one pair per tile: heads and remainders of the split-bf16 inputs
//     accumulate separately, which also gives two independent dependency chains) stay in registers
//     over all K segments; after the last one the four waves' partial tiles meet in LDS, wave
//     t % 4 adds them in a fixed order and runs the epilogue for tile t with all 64 lanes (lane
//     (n = lane % 16, g) holds rows 4g..4g+3 of sequence n: two row pairs).
// Staged input layout (stage_store, XSW form): planes 2n (heads) and 2n+1 (remainders) of nup
// 16-byte units each for sequence n, unit j at index j ^ n, so the 16 sequences read by the lanes of
// one k group fall into different banks.
#pragma once
#include "ff_phases.h"

namespace ff {

constexpr int kDenseMaxTiles = 14;   // tiles of 16 rows one workgroup can own (224 rows: the 70B gate/up projection on 256 workgroups)
constexpr int kDenseSegUnits = kLdsActBytes / (kMaxBatchWide * 8 * 4);   // 16-byte units (8 columns) of one staged K segment
static_assert(kDenseSegUnits == 256 && kDenseSegUnits % kChunkUnitsOf<W_BF16> == 0, "a wide pass's K segment is 2048 columns (64 units per wave, two stages of 32), a whole number of staging chunks");
typedef __bf16 mfma_bf8 __attribute__((ext_vector_type(8)));

struct DenseStream {
    const uint8_t* w; size_t rowb;
    int r0, r1, T;            // rows [r0, r1) of this workgroup; tiles
    int total_units;          // K / 8
    int j0, nunits, nup;      // this K segment: first unit, units, padded units (= kDenseSegUnits)
    bool last, more;          // last segment of the projection / another one follows
    __device__ __forceinline__ static DenseStream make(const PMat& M, int seg, const UDiv& n_ctas) {
        DenseStream D;
        D.w = M.w; D.rowb = (size_t)M.k * 2;
        const u32 ngroups = (u32)(M.n + 3) / 4;
        D.r0 = 4 * (int)n_ctas.div(ngroups * blockIdx.x);
        D.r1 = min(4 * (int)n_ctas.div(ngroups * (blockIdx.x + 1)), M.n);
        D.T = (D.r1 - D.r0 + 15) >> 4;
        D.total_units = M.k / 8;
        D.j0 = seg * kDenseSegUnits;
        D.nunits = min(kDenseSegUnits, D.total_units - D.j0);
        D.nup = kDenseSegUnits;
        D.more = D.j0 + kDenseSegUnits < D.total_units;
        D.last = !D.more;
        return D;
    }
};

// Loads of stage h (0, 1) of tile t in the K segment that starts at unit j0 and holds nunits units.
// Every load is issued from a clamped address: rows past the workgroup's range repeat its last row
// (same addresses within one wave load, i.e. no extra traffic; their results are never stored),
// units past the segment meet zeros in the staged input.
__device__ __forceinline__ void dense_load(const DenseStream& D, int j0, int nunits, int t, int h, Stage<W_BF16>& st, int wave, int lane) {
    const int row = min(D.r0 + 16 * t + (lane & 15), D.r1 - 1);
    const uint8_t* rp = D.w + (size_t)row * D.rowb + (size_t)j0 * 16;
#pragma unroll
    for (int u = 0; u < 8; u++) {
        const int j = min(64 * wave + 32 * h + 4 * u + (lane >> 4), nunits - 1);
        st.w[u >> 2][u & 3] = ldg_stream(rp + (size_t)j * 16);
    }
}

// First two stages of a projection (tile 0 of segment 0), issued before its input is waited for.
__device__ __forceinline__ void dense_prefetch(const DenseStream& D, Stage<W_BF16> (&ring)[2], int wave, int lane) {
    if (D.T > 0) {
        dense_load(D, D.j0, D.nunits, 0, 0, ring[0], wave, lane);
        dense_load(D, D.j0, D.nunits, 0, 1, ring[1], wave, lane);
    }
}

// One K segment of the workgroup's tiles; on the last segment also the reduction over the waves and
// the epilogue.  ah / al: accumulators (zeroed by the caller before segment 0).  epi(pair, b, v0,
// v1) as in gemv_run; post: deferred RMSNorm scale (see PostScale).
template <class Epi>
__device__ __forceinline__ void dense_run(const DenseStream& D, Stage<W_BF16> (&ring)[2], const float4* xs, mfma_f4 (&ah)[kDenseMaxTiles],
                                          mfma_f4 (&al)[kDenseMaxTiles], int batch, int wave, int lane, Epi& epi, const PostScale post) {
    const int n = lane & 15, g = lane >> 4;
    const u32x4* xh = (const u32x4*)xs + (size_t)(2 * n) * D.nup;
    const u32x4* xl = xh + D.nup;
    // The eight k steps of a stage in two groups of four: the group's eight LDS reads are issued
    // together, then its eight matrix-core instructions (a read waited for one at a time would add
    // its latency sixteen times per stage).
    auto compute = [&](const Stage<W_BF16>& st, int h, mfma_f4& ch, mfma_f4& cl) {
#pragma unroll
        for (int u0 = 0; u0 < 8; u0 += 4) {
            u32x4 bh[4], bl[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int j = (64 * wave + 32 * h + 4 * (u0 + u) + g) ^ n;
                bh[u] = xh[j];
                bl[u] = xl[j];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const mfma_bf8 a = __builtin_bit_cast(mfma_bf8, st.w[(u0 + u) >> 2][(u0 + u) & 3]);
                ch = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(mfma_bf8, bh[u]), ch, 0, 0, 0);
                cl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(mfma_bf8, bl[u]), cl, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    const int j0n = D.j0 + kDenseSegUnits, nunitsn = min(kDenseSegUnits, D.total_units - j0n);   // the next segment (if D.more)
#pragma unroll
    for (int t = 0; t < kDenseMaxTiles; t++) {
        if (t < D.T) {
#pragma unroll
            for (int h = 0; h < 2; h++) {
                compute(ring[h], h, ah[t], al[t]);
                __builtin_amdgcn_sched_barrier(0);
                if (t + 1 < D.T) dense_load(D, D.j0, D.nunits, t + 1, h, ring[h], wave, lane);
                else if (D.more) dense_load(D, j0n, nunitsn, 0, h, ring[h], wave, lane);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    if (!D.last) return;
    // ---- the four waves' partial tiles meet in LDS (the staged segment is no longer needed) ----
    __syncthreads();
    float* rb = (float*)xs;   // [T][wave][4][64]
#pragma unroll
    for (int t = 0; t < kDenseMaxTiles; t++) {
        if (t < D.T) {
#pragma unroll
            for (int i = 0; i < 4; i++) rb[((t * kWaves + wave) * 4 + i) * 64 + lane] = ah[t][i] + al[t][i];
        }
    }
    __syncthreads();
    float rs = 1.f;
    if (post.ss) {
        const float* q = post.ss + n;
        rs = rsqrtf(((q[0] + q[kMaxBatchWide]) + (q[2 * kMaxBatchWide] + q[3 * kMaxBatchWide])) * post.inv_k + post.eps);
    }
    for (int t = wave; t < D.T; t += kWaves) {
        float c[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const float* p = rb + ((t * kWaves) * 4 + i) * 64 + lane;
            c[i] = ((p[0] + p[4 * 64]) + (p[8 * 64] + p[12 * 64])) * rs;
        }
        const int row = D.r0 + 16 * t + 4 * g;
        if (n < batch && row < D.r1) {
            epi(row >> 1, n, c[0], c[1]);
            if (row + 2 < D.r1) epi((row >> 1) + 1, n, c[2], c[3]);
        }
    }
}

}  // namespace ff
