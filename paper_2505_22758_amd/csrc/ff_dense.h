// Row partition and weight loads of the wide pass (5..16 sequences, bf16 weights): the projections
// run as a dense contraction on the matrix cores, v_mfma_f32_16x16x32_bf16 multiplying a tile of 16
// weight rows x 32 columns by the inputs of 16 sequences over the same 32 columns.
//
// The paper keeps its row-partitioned matrix-vector scheme up to batch 4 (Section 5.2, larger batch
// sizes) and leaves more sequences open; at 16 sequences the 4x4x4 blocks of gemv_run_quad would
// re-read every staged input once per group of four rows (eight LDS bytes per weight byte).  Here
//   * a WORKGROUP owns a contiguous range of rows (N / workgroups, in groups of four), cut into
//     tiles of 16; its four waves split K: within every staged K segment (2048 columns) wave w
//     multiplies columns [512 w, 512 w + 512) of ALL the workgroup's tiles, so each staged input
//     element is read from LDS once per tile by one wave only (two LDS bytes per weight byte);
//   * lane (r = lane % 16, g = lane / 16) loads 16 bytes of row r of the tile: per wave load 16 rows
//     x 64 contiguous bytes, eight of them (one ring stage) = 512 contiguous bytes per row, two
//     stages per (tile, segment); the same two-stage register ring as the other paths, refilled
//     across tile and segment boundaries.
// The multiply loop, the exchange format and the phase loop are in ff_wide.h.
#pragma once
#include "ff_phases.h"

namespace ff {

constexpr int kDenseMaxTiles = 14;   // tiles of 16 rows one workgroup can own (224 rows: the 70B gate/up projection on 256 workgroups)
constexpr int kDenseSegUnits = kWideSegUnits;   // 16-byte units (8 columns) of one staged K segment: 16 sequences x 2048 columns x (2 + 2) bytes fill the LDS input region
static_assert(kDenseSegUnits == 256 && kDenseSegUnits * kMaxBatchWide * 2 * 16 == kLdsActBytes, "a wide pass's K segment is 2048 columns: 64 units per wave, two stages of 32");
typedef __bf16 mfma_bf8 __attribute__((ext_vector_type(8)));

// K-split projections (output and down projection: few rows per workgroup, so the copies of the
// input images weigh as much as the weights): workgroups 2 p and 2 p + 1 form a pair that multiplies the
// rows of BOTH, each over its half of the K segments, and hands the partner the partial sums of the
// partner's rows (dense_run_wide); every workgroup then reads half the image bytes for the same weight bytes.
constexpr int kWideXchFloats = (kDenseMaxTiles / 2) * 16 * kMaxBatchWide;   // partial sums one workgroup can receive: its own rows (at most half the tiles) x 16 sequences
// Weight formats of the wide pass: bf16 (a 16-byte unit = 8 columns, 256 units per K segment) and
// int8 per-channel (16 columns per unit, 128 units per segment; the codes are converted to bf16 --
// exact -- in registers, the row scales applied to the finished sums), int4 group-128 (32 columns per
// unit, 64 units per segment; see dense_tiles_i4).
template <int WD> constexpr int kDenseSegW = WD == W_BF16 ? kDenseSegUnits : WD == W_INT8 ? kDenseSegUnits / 2 : kDenseSegUnits / 4;   // weight units per K segment
struct DenseStream {
    const uint8_t* w; size_t rowb;
    const f16_t* s;           // int8: row scales; int4: group scales [n][K / 128]
    const f16_t* z;           // int4: group zeros
    int ng;                   // int4: groups per row
    int r0, r1, T;            // rows [r0, r1) this workgroup multiplies (with a K split: the pair's); tiles
    int own0, own1;           // rows it finishes (= [r0, r1) without a K split)
    int seg0, seg1;           // K segments [seg0, seg1) it multiplies
    int total_units;          // weight units per row (K / 8 or K / 16)
    int j0, nunits, nup;      // this K segment: first weight unit, units, padded units
    bool last, more;          // last segment of this workgroup's share / another one follows
    bool split;
    // Is this projection split between the workgroups of a pair?  Even grid, the pair's tiles fit, and an even
    // number of at least four K segments: with fewer (or unequal halves) the hand-over between the partners costs
    // more than the copies it saves (8B shape: output projection 2 segments, down projection 7 -- slower split;
    // 70B shape: 4 and 14 -- 2.5 % faster per step).
    __device__ __forceinline__ static bool can_split(const PMat& M, const UDiv& n_ctas) {
        const u32 ngroups = (u32)(M.n + 3) / 4;
        const int rows_max = 4 * (int)n_ctas.div(ngroups + n_ctas.n - 1u);
        const int nseg = (M.k / 8 + kDenseSegUnits - 1) / kDenseSegUnits;
        return (n_ctas.n & 1u) == 0 && nseg >= 4 && (nseg & 1) == 0 && 2 * rows_max <= kDenseMaxTiles * 16;
    }
    template <int WD = W_BF16>
    __device__ __forceinline__ static DenseStream make(const PMat& M, int seg, const UDiv& n_ctas, bool split = false) {
        constexpr int SEGW = kDenseSegW<WD>;
        DenseStream D;
        D.w = M.w; D.s = M.s; D.z = M.z; D.ng = M.k / 128;
        D.rowb = WD == W_BF16 ? (size_t)M.k * 2 : WD == W_INT8 ? (size_t)M.k : (size_t)M.k / 2;
        const u32 ngroups = (u32)(M.n + 3) / 4;
        D.own0 = 4 * (int)n_ctas.div(ngroups * blockIdx.x);
        D.own1 = min(4 * (int)n_ctas.div(ngroups * (blockIdx.x + 1)), M.n);
        D.total_units = M.k / (WD == W_BF16 ? 8 : WD == W_INT8 ? 16 : 32);
        const int nseg = (D.total_units + SEGW - 1) / SEGW;
        D.split = split;
        if (split) {
            const u32 p = blockIdx.x & ~1u;
            D.r0 = 4 * (int)n_ctas.div(ngroups * p);
            D.r1 = min(4 * (int)n_ctas.div(ngroups * (p + 2)), M.n);
            const int half = (nseg + 1) / 2;
            D.seg0 = (blockIdx.x & 1) ? half : 0;
            D.seg1 = (blockIdx.x & 1) ? nseg : half;
        } else {
            D.r0 = D.own0; D.r1 = D.own1; D.seg0 = 0; D.seg1 = nseg;
        }
        D.T = (D.r1 - D.r0 + 15) >> 4;
        D.j0 = seg * SEGW;
        D.nunits = min(SEGW, D.total_units - D.j0);
        D.nup = SEGW;
        D.more = seg + 1 < D.seg1;
        D.last = !D.more;
        return D;
    }
};

// Loads of stage h (0, 1) of tile t in the K segment that starts at unit j0 and holds nunits units.
// Every load is issued from a clamped address: rows past the workgroup's range repeat its last row
// (same addresses within one wave load, i.e. no extra traffic; their results are never stored),
// units past the segment meet zeros in the staged input.  With `real` false (no further stage in the
// projection) the eight loads are still issued, all lanes reading the matrix's first 16 bytes: the
// number of loads in flight then never depends on a branch, which is what lets the compiler wait for
// a ring slot with the other slot's loads still outstanding (where code paths that issued different
// numbers of loads meet, it has to assume the fewest, i.e. wait for everything).
__device__ __forceinline__ void dense_load(const DenseStream& D, int j0, int nunits, int t, int h, Stage<W_BF16>& st, int wave, int lane, bool real = true) {
    const int row = min(D.r0 + 16 * t + (lane & 15), D.r1 - 1);
    const uint8_t* rp = D.w + (size_t)row * D.rowb + (size_t)j0 * 16;
#pragma unroll
    for (int u = 0; u < 8; u++) {
        const int j = min(64 * wave + 32 * h + 4 * u + (lane >> 4), nunits - 1);
        st.w[u >> 2][u & 3] = ldg_stream(real ? rp + (size_t)j * 16 : D.w);
    }
}

// int8: a wave's K quarter of a segment is 32 units of 16 columns = ONE stage of eight loads per tile (lane (r, g):
// unit 32 w + 4 u + g of row r).  The stream of stages then runs segment by segment, tile by tile, and the cursor of
// the next stage to load is carried from stage to stage.
struct DenseCursor {
    int seg, t;
    __device__ __forceinline__ void advance(int T) {   // (selects, not branches)
        const int wt = t + 1 >= T ? 1 : 0;
        t = wt ? 0 : t + 1;
        seg += wt;
    }
};
__device__ __forceinline__ void dense_load_i8(const DenseStream& D, const DenseCursor& c, Stage<W_INT8>& st, int wave, int lane) {
    constexpr int SEGW = kDenseSegW<W_INT8>;
    const bool real = c.seg < D.seg1;   // behind the last stage: eight loads of one address (see dense_load)
    const int row = min(D.r0 + 16 * c.t + (lane & 15), D.r1 - 1);
    const uint8_t* rp = D.w + (size_t)row * D.rowb + (size_t)c.seg * (SEGW * 16);
    const int jmax = D.total_units - c.seg * SEGW - 1;
#pragma unroll
    for (int u = 0; u < 8; u++) {
        const int j = min(32 * wave + 4 * u + (lane >> 4), jmax);
        st.w[u >> 2][u & 3] = ldg_stream(real ? rp + (size_t)j * 16 : D.w);
    }
}
__device__ __forceinline__ void dense_prefetch_i8(const DenseStream& D, DenseCursor& c, Stage<W_INT8> (&ring)[2], int wave, int lane) {
    c = DenseCursor{D.seg0, 0};
    if (D.T > 0) {
        dense_load_i8(D, c, ring[0], wave, lane);
        c.advance(D.T);
        dense_load_i8(D, c, ring[1], wave, lane);
        c.advance(D.T);
    }
}

// int4: a unit is 32 columns of ONE group of 128; a wave's K quarter of a segment is 16 units = four groups, lane
// (r, g) loading unit 16 w + 4 u + g of row r (u = 0..3: the four lanes g of a row hold the four units of group u).
// That is four loads per tile, so a ring stage covers a PAIR of tiles (2 tp, 2 tp + 1: eight loads; the second
// tile of the last pair may not exist -- its loads are then dummies), plus per tile the row's scales and zeros of the
// quarter's four groups (8 bytes each).  Needs K to be a multiple of 512 (whole quarters of groups), which the host checks.
struct WideStageI4 {
    u32x4 w[2][4];     // [tile of the pair][u]
    u32x2 s[2], z[2];  // raw fp16 scales / zeros of row r, groups 4 w .. 4 w + 3 of the segment
};
__device__ __forceinline__ void dense_load_i4(const DenseStream& D, const DenseCursor& c, WideStageI4& st, int wave, int lane) {
    constexpr int SEGW = kDenseSegW<W_INT4>;
    const bool real = c.seg < D.seg1;   // behind the last stage: loads of one address (see dense_load)
#pragma unroll
    for (int k = 0; k < 2; k++) {
        const int t = 2 * c.t + k;   // (c.t counts tile pairs)
        const bool rt = real && t < D.T;
        const int row = min(D.r0 + 16 * t + (lane & 15), D.r1 - 1);
        const uint8_t* rp = D.w + (size_t)row * D.rowb + (size_t)c.seg * (SEGW * 16);
        const int jmax = D.total_units - c.seg * SEGW - 1;   // units past the end of K are clamped (they meet zeros in the staged input)
#pragma unroll
        for (int u = 0; u < 4; u++) st.w[k][u] = ldg_stream(rt ? rp + (size_t)min(16 * wave + 4 * u + (lane >> 4), jmax) * 16 : D.w);
        const size_t gi = (size_t)row * D.ng + (size_t)min(c.seg * (SEGW / 4) + 4 * wave, D.ng - 4);   // (likewise the groups: ng is a multiple of four)
        st.s[k] = *as_global((const u32x2*)(rt ? D.s + gi : D.s));
        st.z[k] = *as_global((const u32x2*)(rt ? D.z + gi : D.z));
    }
}
__device__ __forceinline__ void dense_prefetch_i4(const DenseStream& D, DenseCursor& c, WideStageI4 (&ring)[2], int wave, int lane) {
    c = DenseCursor{D.seg0, 0};
    if (D.T > 0) {
        const int TP = (D.T + 1) >> 1;
        dense_load_i4(D, c, ring[0], wave, lane);
        c.advance(TP);
        dense_load_i4(D, c, ring[1], wave, lane);
        c.advance(TP);
    }
}
template <int WD> struct WideStageOf { typedef Stage<WD> type; };
template <> struct WideStageOf<W_INT4> { typedef WideStageI4 type; };

// First two stages of a projection (tile 0 of segment 0), issued before its input is waited for.
__device__ __forceinline__ void dense_prefetch(const DenseStream& D, Stage<W_BF16> (&ring)[2], int wave, int lane) {
    if (D.T > 0) {
        dense_load(D, D.j0, D.nunits, 0, 0, ring[0], wave, lane);
        dense_load(D, D.j0, D.nunits, 0, 1, ring[1], wave, lane);
    }
}

}  // namespace ff
