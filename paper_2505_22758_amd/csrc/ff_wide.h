// The wide pass (9..16 sequences, bf16 weights): exchange between workgroups and the phase loop.
//
// Up to eight sequences every workgroup stages every sequence's whole input itself (load the tagged
// words, add the sublayer output, normalise, convert to the matrix cores' head/remainder form).  At
// 16 sequences that conversion alone costs more than half of what streaming the weights costs
// (16 x 70 K values per layer and workgroup at the 70B shape), all of it replicated 256 times.  The
// wide pass therefore exchanges activations in the form their consumers multiply, produced once by
// the workgroup that OWNS the value:
//   * every workgroup owns a fixed range of rows of the residual stream (the rows of the output
//     and down projections it computes, N / workgroups) and keeps them in a plain buffer of its
//     own; the epilogue of those two projections adds the projection output to its rows, and writes
//     (gain of the next normalised projection) x (new value) as bf16 head + bf16 remainder straight
//     into a global IMAGE of the consumers' LDS layout, plus the workgroup's share of every
//     sequence's sum of squares (the 1/rms factor is applied by the consumer to its finished sums:
//     a scalar per sequence that commutes with the projection);
//   * the SwiGLU epilogue and the attention merge write their outputs into such images too;
//   * a consumer's staging is a copy: image segment (2048 columns x 16 sequences, 128 KB) -> LDS,
//     16 bytes per lane and instruction, no arithmetic, each wave copying the K quarter it multiplies
//     (no workgroup barrier between segments);
//   * the image words have no room for the per-word write counters of the other paths, so the
//     dependency is carried by one flag per workgroup and phase (paper Section 4.1: the global
//     barrier between dependent phases, here as an epoch per workgroup that consumers poll): a
//     producer makes its exchange stores (all write-through, agent scope), waits until they have
//     completed, and publishes the phase's epoch; a consumer polls until all workgroups show the
//     epoch, drops cached copies of earlier contents (agent-scope acquire) and reads with plain
//     cacheable loads, which the workgroups of an XCD serve each other out of their L2.
//     Queries, keys, values and attention partials keep their tagged 8-byte format.
// Write-after-read on the images is ordered by the same epochs (an image is rewritten only by
// workgroups that have waited for an epoch which every reader of the old contents published after
// its last read).
#pragma once
#include "ff_dense.h"

namespace ff {

__host__ __device__ inline size_t wide_img_bytes(int K) { return (size_t)((K + 2047) / 2048) * kWideSegBytes; }

// ---------------------------------------------------------------- epochs
struct WideSync {
    u32* flags;       // [workgroups] last epoch each workgroup has published
    int ncta;
    lds_u32* ok_slot; // LDS word for the verdict
    u32* pflags;      // [workgroups] last epoch whose partial sums each workgroup has handed to its partner (K-split projections)
    // This workgroup's partial sums for its partner are stored: publish.
    __device__ __forceinline__ void arrive_pair(u32 epoch) const {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0) xst_u32(pflags + blockIdx.x, epoch);
    }
    // The partner has published `epoch`.  Its sums are read with coherent loads, so no fence here.  False (uniformly) on a time-out.
    __device__ __forceinline__ bool wait_pair(u32 epoch, int wave, int lane) const {
        if (wave == 0) {
            bool ok = false;
            for (int spins = 0; spins < kSpinLimit && !ok; spins++) {
                ok = (int)(xld_u32(pflags + (blockIdx.x ^ 1u)) - epoch) >= 0;
                if (!ok) __builtin_amdgcn_s_sleep(2);
            }
            if (lane == 0) *ok_slot = ok ? 1u : 0u;
        }
        __syncthreads();
        const bool ok = *ok_slot != 0u;
        __syncthreads();
        return ok;
    }
    // All of this workgroup's exchange stores of the phase are made: publish the epoch.
    __device__ __forceinline__ void arrive(u32 epoch) const {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's write-through stores have completed
        __syncthreads();
        if (threadIdx.x == 0) xst_u32(flags + blockIdx.x, epoch);
    }
    // Every workgroup has published `epoch` (or a later one).  Returns false (uniformly) on a time-out.
    __device__ __forceinline__ bool wait(u32 epoch, int wave, int lane) const {
        if (wave == 0) {
            bool ok = false;
            for (int spins = 0; spins < kSpinLimit && !ok; spins++) {
                bool mine = true;
                for (int i = lane; i < ncta; i += 64) mine = mine && (int)(xld_u32(flags + i) - epoch) >= 0;
                ok = __all(mine);
                if (!ok) __builtin_amdgcn_s_sleep(4);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // cached copies of the images' earlier contents are dropped
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (lane == 0) *ok_slot = ok ? 1u : 0u;
        }
        __syncthreads();
        const bool ok = *ok_slot != 0u;
        __syncthreads();   // (the slot is rewritten by the next wait)
        return ok;
    }
};

// ---------------------------------------------------------------- consumer side
// Copies this wave's quarter of one image segment into LDS (same layout): units [64 w, 64 w + 64) of
// the two planes of each of the pass's sequences, one 16-byte unit per lane and plane.  A wave
// multiplies only its own K quarter of a segment (and the unit swizzle j ^ n stays inside a quarter),
// so the copy is private to the wave: no workgroup barrier between K segments, the waves of a
// workgroup drift apart and one wave's copy overlaps the others' weight streams.  The copy uses the
// loads that write LDS directly (global_load_lds_dwordx4: lane i's 16 bytes land at M0 base + 16 i),
// so all planes are requested at once without passing through registers, and one wait covers them.
// The planes of sequences beyond the pass's batch are not copied: their matrix-core columns are never
// stored.  The compiler does not order LDS reads against these loads by itself: the caller's last
// reads of the old contents are complete (their results have been multiplied), and nothing is moved
// across the wait at the end.
__device__ __forceinline__ void wide_copy_quarter(const uint8_t* img_seg, uint8_t* lds, int wave, int lane, int batch) {
    typedef __attribute__((address_space(1))) const void gvoid;
    typedef __attribute__((address_space(3))) void lvoid;
    constexpr int kPlaneBytes = kDenseSegUnits * 16;
    const uint8_t* src = img_seg + (size_t)(64 * wave + lane) * 16;
    uint8_t* dst = lds + (size_t)(64 * wave) * 16;   // wave-uniform
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int n = 0; n < kMaxBatchWide; n++) {
        if (n < batch) {
            __builtin_amdgcn_global_load_lds((gvoid*)(src + (2 * n) * kPlaneBytes), (lvoid*)(dst + (2 * n) * kPlaneBytes), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gvoid*)(src + (2 * n + 1) * kPlaneBytes), (lvoid*)(dst + (2 * n + 1) * kPlaneBytes), 16, 0, 0);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}
// 1/rms of every sequence from the workgroups' partial sums of squares ([workgroups][16] floats,
// added in a fixed order) into rs[16] (LDS).  part: LDS scratch of 256 floats.
__device__ __forceinline__ void wide_rms(const float* sspart, int ncta, int K, float eps, float* part, float* rs, int tid) {
    const int n = tid & 15, grp = tid >> 4;   // 16 groups of workgroups
    // (all loads of a thread are issued before the first is added: one trip to the L2 instead of sixteen;
    // a wide pass runs on at most 256 workgroups, which the host checks when the model is created)
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = as_global(sspart)[min(grp + 16 * i, ncta - 1) * kMaxBatchWide + n];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i++) s += grp + 16 * i < ncta ? v[i] : 0.f;
    part[grp * 16 + n] = s;
    __syncthreads();
    if (tid < 16) {
        float t = 0.f;
#pragma unroll
        for (int gI = 0; gI < 16; gI++) t += part[gI * 16 + tid];
        rs[tid] = rsqrtf(t / (float)K + eps);
    }
    __syncthreads();
}

// ---------------------------------------------------------------- producer side (epilogues)
// Called by dense_run_wide for lane (n = sequence, rows row .. row+3 of the projection, nv of them
// inside the workgroup's range: 2 or 4) with the finished sums c[0..3].
template <class E>
struct WideEpiPairs {   // projections whose epilogue works on row pairs (QKV: RoPE + cache append; LM head)
    E& e;
    __device__ __forceinline__ void operator()(int row, int n, const float (&c)[4], int nv) const {
        e(row >> 1, n, c[0], c[1]);
        if (nv > 2) e((row >> 1) + 1, n, c[2], c[3]);
    }
};
struct WideEpiSwiGLU {   // gate/up pairs -> h = silu(gate) * up into the image of the down projection's input
    uint8_t* img; GuPerm perm;
    __device__ __forceinline__ void operator()(int row, int n, const float (&c)[4], int nv) const {
#pragma unroll
        for (int p = 0; p < 2; p++) {
            if (2 * p < nv) {
                const float g = c[2 * p], u = c[2 * p + 1];
                const float h = g / (1.0f + expf(-g)) * u;
                u32 hi, lo;
                split_bf16x2(h, 0.f, hi, lo);
                const int f = perm.unit_of_pair((row >> 1) + p);
                __hip_atomic_store(as_global((uint16_t*)(img + wide_img_off(n, 0, f))), (uint16_t)hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(as_global((uint16_t*)(img + wide_img_off(n, 1, f))), (uint16_t)lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
};
struct WideEpiResidual {   // output / down projection: residual rows of this workgroup += output; image of gain * new value
    float* xres; int d;          // residual stream [16][d] (rows owned by this workgroup only are touched)
    const bf16_t* gain;          // gain of the next normalised projection
    uint8_t* img;                // its input image
    float* ssl;                  // LDS: this workgroup's partial sums of squares, [slot][16]
    int r0;
    __device__ __forceinline__ void operator()(int row, int n, const float (&c)[4], int nv) const {
        // (rows come in whole groups of four here: d is a multiple of 4)
        FF_GLOBAL f32x4* xp = as_global((f32x4*)(xres + (size_t)n * d + row));
        const u32x2 gw = *as_global((const u32x2*)(gain + row));
        f32x4 x = *xp;
        x.x += c[0]; x.y += c[1]; x.z += c[2]; x.w += c[3];
        *xp = x;
        ssl[((row - r0) >> 2) * kMaxBatchWide + n] = (x.x * x.x + x.y * x.y) + (x.z * x.z + x.w * x.w);
        u32 h0, l0, h1, l1;
        split_bf16x2(x.x * bf_lo(gw.x), x.y * bf_hi(gw.x), h0, l0);
        split_bf16x2(x.z * bf_lo(gw.y), x.w * bf_hi(gw.y), h1, l1);
        xst2((float*)(img + wide_img_off(n, 0, row)), __uint_as_float(h0), __uint_as_float(h1));
        xst2((float*)(img + wide_img_off(n, 1, row)), __uint_as_float(l0), __uint_as_float(l1));
    }
};

// One K segment of the workgroup's tiles like dense_run, with the per-sequence 1/rms factors in
// LDS (rs, or null) and an epilogue on groups of four rows (see the epilogue structs above).
// With a K split (D.split) the finished tiles cover the rows of both workgroups of the pair over this
// workgroup's K segments: the sums of the partner's rows go to the partner (xch: [workgroup][group of
// four rows][sequence][4], write-through stores, then the pair flag), the sums of the own rows wait
// for the partner's share and then take the epilogue.  Returns false after a time-out.
// int8: the tiles of one K segment, one ring stage each.  The slot of tile t is (t + PAR) mod 2 with PAR = (stages
// before this segment) mod 2; the tile loop is unrolled, so PAR is static, and the early exit is tested only where
// a T of parity TP can end: all exits of one form leave the ring in the same state (the compiler keeps track of the
// loads in flight per code path and assumes the worst where paths meet).  A lane's 16 codes are two k-steps: codes
// 0..7 against input unit 2 J, codes 8..15 against unit 2 J + 1 (J = 32 w + 4 u + g: the unit's index in the segment).
template <int PAR, int TP>
__device__ __forceinline__ void dense_tiles_i8(const DenseStream& D, Stage<W_INT8> (&ring)[2], const float4* xs, mfma_f4 (&acc)[kDenseMaxTiles],
                                               DenseCursor& cur, int wave, int lane) {
    const int n = lane & 15, g = lane >> 4;
    const u32x4* xh = (const u32x4*)xs + (size_t)(2 * n) * kDenseSegUnits;
    const u32x4* xl = xh + kDenseSegUnits;
    auto pack = [](float lo, float hi) { return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u); };   // upper halves of two floats: a signed byte is exact in bf16
    auto codes = [&](u32 wa, u32 wb) {
        const u32x4 v{pack((float)(int)(int8_t)wa, (float)(int)(int8_t)(wa >> 8)), pack((float)(int)(int8_t)(wa >> 16), (float)((int)wa >> 24)),
                      pack((float)(int)(int8_t)wb, (float)(int)(int8_t)(wb >> 8)), pack((float)(int)(int8_t)(wb >> 16), (float)((int)wb >> 24))};
        return __builtin_bit_cast(mfma_bf8, v);
    };
#pragma unroll
    for (int t = 0; t < kDenseMaxTiles; t++) {
        if ((t & 1) == TP && t >= D.T) break;
        Stage<W_INT8>& st = ring[(t + PAR) & 1];
        mfma_f4& cc = acc[t];
#pragma unroll
        for (int u0 = 0; u0 < 8; u0 += 2) {
            u32x4 bh[4], bl[4];
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const int j = 2 * (32 * wave + 4 * (u0 + u) + g);
                bh[2 * u] = xh[j ^ n]; bl[2 * u] = xl[j ^ n];
                bh[2 * u + 1] = xh[(j + 1) ^ n]; bl[2 * u + 1] = xl[(j + 1) ^ n];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const u32x4 w = st.w[(u0 + u) >> 2][(u0 + u) & 3];
                const mfma_bf8 a0 = codes(w.x, w.y), a1 = codes(w.z, w.w);
                cc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, __builtin_bit_cast(mfma_bf8, bh[2 * u]), cc, 0, 0, 0);
                cc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, __builtin_bit_cast(mfma_bf8, bl[2 * u]), cc, 0, 0, 0);
                cc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, __builtin_bit_cast(mfma_bf8, bh[2 * u + 1]), cc, 0, 0, 0);
                cc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, __builtin_bit_cast(mfma_bf8, bl[2 * u + 1]), cc, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        dense_load_i8(D, cur, st, wave, lane);   // the stage two further on (always eight loads)
        cur.advance(D.T);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// int4 group-128: the tiles of one K segment, one ring stage per PAIR of tiles (see dense_load_i4); slots and exits
// as in dense_tiles_i8, counted in tile pairs (PAR = (stages before this segment) mod 2, TP = (tile pairs) mod 2).
// A wave's quarter of the segment is four groups u = 0..3 of 128 columns; the four lanes g of a row hold the four
// units of a group, so the four k-steps q = 0..3 of one group (codes 8 q .. 8 q + 7 of every lane's unit against
// input unit 4 J + q) sum exactly that group:  with the codes n turned into the bf16 numbers 128 + n by bit
// operations (0x4300 | n), a group yields d = sum (128 + n) x per (row, sequence), and with X = sum of the
// group's x per sequence
//     sum s (n - z) x  =  s (d - (128 + z) X).
// X comes from the same matrix-core instructions with an A operand of ones (once per segment and group: every
// row of that product is X).  Scale s and zero z belong to the ROW: they are loaded by the lanes that load the row's
// codes (lane (r, g): row r, the quarter's four groups) and fetched into the accumulator layout (lane (n, g):
// rows 4 g + i) with one cross-lane read per row and group.
template <int PAR, int TP>
__device__ __forceinline__ void dense_tiles_i4(const DenseStream& D, WideStageI4 (&ring)[2], const float4* xs, mfma_f4 (&acc)[kDenseMaxTiles],
                                               DenseCursor& cur, int wave, int lane) {
    const int n = lane & 15, g = lane >> 4;
    const u32x4* xh = (const u32x4*)xs + (size_t)(2 * n) * kDenseSegUnits;
    const u32x4* xl = xh + kDenseSegUnits;
    const int TPn = (D.T + 1) >> 1;
    // input units of group u, k-step q for this lane: 4 (16 w + 4 u + g) + q
    auto xunit = [&](int u, int q) { return (4 * (16 * wave + 4 * u + g) + q) ^ n; };
    // X[u] = sum of the group's inputs of sequence n (same in every lane (n, .))
    float X[4];
    {
        const u32x4 ones{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
#pragma unroll
        for (int u = 0; u < 4; u++) {
            mfma_f4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const u32x4 bh = xh[xunit(u, q)], bl = xl[xunit(u, q)];
                c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(mfma_bf8, ones), __builtin_bit_cast(mfma_bf8, bh), c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(mfma_bf8, ones), __builtin_bit_cast(mfma_bf8, bl), c, 0, 0, 0);
            }
            X[u] = c[0];
        }
    }
    auto codes = [](u32 w) {   // eight codes of one word as bf16 128 + n, in column order
        const u32 e = w & 0x0F0F0F0Fu, o = (w >> 4) & 0x0F0F0F0Fu;   // codes 0,2,4,6 / 1,3,5,7 as bytes
        const u32x4 v{__builtin_amdgcn_perm(o, e, 0x0c040c00u) | 0x43004300u, __builtin_amdgcn_perm(o, e, 0x0c050c01u) | 0x43004300u,
                      __builtin_amdgcn_perm(o, e, 0x0c060c02u) | 0x43004300u, __builtin_amdgcn_perm(o, e, 0x0c070c03u) | 0x43004300u};
        return __builtin_bit_cast(mfma_bf8, v);
    };
    // two k-steps of one group of one tile
    auto steps2 = [&](const u32x4& w, int q0, const u32x4 (&bh)[2], const u32x4 (&bl)[2], mfma_f4& d) {
        const u32 ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int q = 0; q < 2; q++) {
            const mfma_bf8 a = codes(ww[q0 + q]);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(mfma_bf8, bh[q]), d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(mfma_bf8, bl[q]), d, 0, 0, 0);
        }
    };
    // the group's contribution with the rows' scales and zeros: those of rows 4 g + i are held by lane 4 g + i
    auto combine = [&](u32 sbits, u32 zbits, float Xu, const mfma_f4& d, mfma_f4& cc) {
        const u32 szp = sbits | (zbits << 16);
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const u32 v = (u32)__builtin_amdgcn_ds_bpermute((4 * g + i) * 4, (int)szp);
            const float sc = f16_to_f((f16_t)(v & 0xFFFFu)), zp = 128.f + f16_to_f((f16_t)(v >> 16));
            cc[i] = fmaf(sc, fmaf(-zp, Xu, d[i]), cc[i]);
        }
    };
    auto half16 = [](const u32x2& v, int u) { const u32 w = u < 2 ? v.x : v.y; return (u & 1) ? w >> 16 : w & 0xFFFFu; };
#pragma unroll
    for (int tp = 0; tp < (kDenseMaxTiles + 1) / 2; tp++) {
        if ((tp & 1) == TP && tp >= TPn) break;
        WideStageI4& st = ring[(tp + PAR) & 1];
        const bool two = 2 * tp + 1 < D.T;
        mfma_f4& c0 = acc[2 * tp];
        mfma_f4& c1 = acc[2 * tp + 1 < kDenseMaxTiles ? 2 * tp + 1 : 0];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            mfma_f4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q0 = 0; q0 < 4; q0 += 2) {
                u32x4 bh[2], bl[2];   // the inputs of two k-steps: shared by the two tiles of the pair
#pragma unroll
                for (int q = 0; q < 2; q++) { bh[q] = xh[xunit(u, q0 + q)]; bl[q] = xl[xunit(u, q0 + q)]; }
                __builtin_amdgcn_sched_barrier(0);
                steps2(st.w[0][u], q0, bh, bl, d0);
                if (two) steps2(st.w[1][u], q0, bh, bl, d1);
                __builtin_amdgcn_sched_barrier(0);
            }
            combine(half16(st.s[0], u), half16(st.z[0], u), X[u], d0, c0);
            if (two) combine(half16(st.s[1], u), half16(st.z[1], u), X[u], d1, c1);
            __builtin_amdgcn_sched_barrier(0);
        }
        dense_load_i4(D, cur, st, wave, lane);   // the stage two further on (always the same number of loads)
        cur.advance(TPn);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int WD, class Epi>
__device__ __forceinline__ bool dense_run_wide(const DenseStream& D, typename WideStageOf<WD>::type (&ring)[2], const float4* xs, mfma_f4 (&acc)[kDenseMaxTiles],
                                               int batch, int wave, int lane, const Epi& epi, const float* rs_lds,
                                               float* xch = nullptr, const WideSync* sync = nullptr, u32 pepoch = 0, DenseCursor* cur = nullptr, int par = 0) {
    const int n = lane & 15, g = lane >> 4;
  if constexpr (WD == W_INT4) {
    if (((D.T + 1) >> 1) & 1) {
        if (par) dense_tiles_i4<1, 1>(D, ring, xs, acc, *cur, wave, lane);
        else dense_tiles_i4<0, 1>(D, ring, xs, acc, *cur, wave, lane);
    } else dense_tiles_i4<0, 0>(D, ring, xs, acc, *cur, wave, lane);
  } else if constexpr (WD == W_INT8) {
    if (D.T & 1) {
        if (par) dense_tiles_i8<1, 1>(D, ring, xs, acc, *cur, wave, lane);
        else dense_tiles_i8<0, 1>(D, ring, xs, acc, *cur, wave, lane);
    } else dense_tiles_i8<0, 0>(D, ring, xs, acc, *cur, wave, lane);
  } else {
    const u32x4* xh = (const u32x4*)xs + (size_t)(2 * n) * kDenseSegUnits;
    const u32x4* xl = xh + kDenseSegUnits;
    auto compute = [&](const Stage<W_BF16>& st, int h, mfma_f4& cc) {
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
                cc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(mfma_bf8, bh[u]), cc, 0, 0, 0);
                cc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(mfma_bf8, bl[u]), cc, 0, 0, 0);
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
                compute(ring[h], h, acc[t]);
                __builtin_amdgcn_sched_barrier(0);
                // (the next tile's stage, the next segment's first, or a dummy: always eight loads, see dense_load)
                const bool in_seg = t + 1 < D.T;
                dense_load(D, in_seg ? D.j0 : j0n, in_seg ? D.nunits : nunitsn, in_seg ? t + 1 : 0, h, ring[h], wave, lane, in_seg || D.more);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
  }
    if (!D.last) return true;
    // ---- the four waves' partial tiles meet in LDS (the staged segment is no longer needed) ----
    __syncthreads();
    float* rb = (float*)xs;   // [T][wave][4][64]
#pragma unroll
    for (int t = 0; t < kDenseMaxTiles; t++) {
        if (t < D.T) {
#pragma unroll
            for (int i = 0; i < 4; i++) rb[((t * kWaves + wave) * 4 + i) * 64 + lane] = acc[t][i];
        }
    }
    __syncthreads();
    const float rs = rs_lds ? rs_lds[n] : 1.f;
    auto tile_sums = [&](int t, float (&c)[4]) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const float* p = rb + ((t * kWaves) * 4 + i) * 64 + lane;
            c[i] = ((p[0] + p[4 * 64]) + (p[8 * 64] + p[12 * 64])) * rs;
            if constexpr (WD == W_INT8) c[i] *= f16_to_f(as_global(D.s)[min(D.r0 + 16 * t + 4 * g + i, D.r1 - 1)]);   // row scale
        }
    };
    if (!D.split) {
        for (int t = wave; t < D.T; t += kWaves) {
            float c[4];
            tile_sums(t, c);
            const int row = D.r0 + 16 * t + 4 * g;
            if (n < batch && row < D.r1) epi(row, n, c, min(4, D.r1 - row));
        }
        return true;
    }
    // ---- K split: the partner's rows first, so that it can go on ----
    const bool second = (blockIdx.x & 1u) != 0;
    const int p0 = second ? D.r0 : D.own1, p1 = second ? D.own0 : D.r1;   // the partner's rows
    float* xout = xch + (size_t)(blockIdx.x ^ 1u) * kWideXchFloats;
    for (int t = wave; t < D.T; t += kWaves) {
        const int row = D.r0 + 16 * t + 4 * g;
        if (n < batch && row >= p0 && row < p1) {
            float c[4];
            tile_sums(t, c);
            float* q = xout + ((size_t)((row - p0) >> 2) * kMaxBatchWide + n) * 4;
            xst2(q, c[0], c[1]);
            xst2(q + 2, c[2], c[3]);
        }
    }
    sync->arrive_pair(pepoch);
    if (!sync->wait_pair(pepoch, wave, lane)) return false;
    const float* xin = xch + (size_t)blockIdx.x * kWideXchFloats;
    for (int t = wave; t < D.T; t += kWaves) {
        const int row = D.r0 + 16 * t + 4 * g;
        if (n < batch && row >= D.own0 && row < D.own1) {
            float c[4];
            tile_sums(t, c);
            const float* q = xin + ((size_t)((row - D.own0) >> 2) * kMaxBatchWide + n) * 4;
            const u64 a = __hip_atomic_load(as_global((const u64*)q), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const u64 b = __hip_atomic_load(as_global((const u64*)(q + 2)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c[0] += __uint_as_float((u32)a); c[1] += __uint_as_float((u32)(a >> 32));
            c[2] += __uint_as_float((u32)b); c[3] += __uint_as_float((u32)(b >> 32));
            epi(row, n, c, min(4, D.own1 - row));
        }
    }
    return true;
}

}  // namespace ff
