// Kernels: the fused whole-model decode step, the per-operation baseline, and the loaders.
#pragma once
#include "ff_phases.h"

namespace ff {

// status codes written by kernels (mirror the C ABI's FF_ERR_*)
constexpr int kStatusRange = -3;
constexpr int kStatusTimeout = -5;

__device__ __forceinline__ bool inputs_ok(const DevModel& M, const DevKV& KV, const int* tokens, const int* pos, int batch) {
    bool ok = true;
    for (int b = 0; b < batch; b++) {
        int p = pos[b], t = tokens[b];
        ok = ok && p >= 0 && p < KV.max_ctx && t >= 0 && t < M.V;
    }
    return ok;
}

// Device-wide barrier among the gridDim.x co-resident workgroups of the fused kernel (paper
// Section 3.1, global memory ordering: an atomic-based global synchronisation coupled with each
// thread completing its own global writes first).  Every workgroup publishes the generation it
// has reached in its own flag word; everyone polls all flags.  No read-modify-write, so arrivals
// do not serialise on one address.  Exchange data is written with coherent (agent-scope) stores
// before the flag and read with coherent loads after it, so no cache maintenance is needed.
// Returns false (and records a time-out) if the other workgroups never arrive.
__device__ __forceinline__ bool grid_barrier(const DevModel& M, u32 gen) {
    __builtin_amdgcn_s_waitcnt(0);   // this thread's stores have been acknowledged
    __syncthreads();
    if (threadIdx.x == 0) xst_u32(&M.bar_flags[blockIdx.x], gen);
    for (int spins = 0; spins < kSpinLimit; spins++) {
        bool mine = true;
        for (int c = threadIdx.x; c < (int)gridDim.x; c += kThreads)
            mine = mine && (int)(xld_u32(&M.bar_flags[c]) - gen) >= 0;
        if (__syncthreads_and(mine)) return true;
    }
    if (threadIdx.x == 0) atomicExch(M.status, kStatusTimeout);
    return false;
}

template <class IO>
__device__ void attention_phase(const DevModel& M, const DevKV& KV, const int* pos, int batch, int layer, uint8_t* lds,
                                bool fused_merge) {
    const int G = M.Hq / M.Hkv;
    const int share = max(1, (int)gridDim.x / (batch * M.Hkv));
    int base = 0;
    __shared__ u32 s_old;
    for (int b = 0; b < batch; b++) {
        const int T = pos[b];
        const int ns = attn_nsplit(T, share);
        const int nitems = M.Hkv * ns;
        // items of sequence b occupy [base, base + nitems) of the global item list
        int first = ((int)blockIdx.x - base) % (int)gridDim.x;
        if (first < 0) first += gridDim.x;
        for (int it = first; it < nitems; it += gridDim.x) {
            int j = it / ns, s = it % ns;
            int t0 = (int)((long)T * s / ns), t1 = (int)((long)T * (s + 1) / ns);
            bool cur = s == ns - 1;
            if (M.hd == 64 && G == 4) attn_item<64, 4, IO>(M, KV, layer, b, j, t0, t1, cur, s, lds);
            else if (M.hd == 128 && G == 4) attn_item<128, 4, IO>(M, KV, layer, b, j, t0, t1, cur, s, lds);
            else if (M.hd == 128 && G == 8) attn_item<128, 8, IO>(M, KV, layer, b, j, t0, t1, cur, s, lds);
            if (fused_merge) {
                // last workgroup to finish a split of (b, j) merges all of them
                __builtin_amdgcn_s_waitcnt(0);
                __syncthreads();
                if (threadIdx.x == 0)
                    s_old = __hip_atomic_fetch_add(&M.head_ctr[b * M.Hkv + j], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __syncthreads();
                if ((s_old + 1) % (u32)ns == 0) {
                    if (M.hd == 64 && G == 4) attn_merge<64, 4, IO>(M, b, j, ns);
                    else if (M.hd == 128 && G == 4) attn_merge<128, 4, IO>(M, b, j, ns);
                    else if (M.hd == 128 && G == 8) attn_merge<128, 8, IO>(M, b, j, ns);
                }
            }
        }
        base = (base + nitems) % (int)gridDim.x;
    }
}

// ---------------------------------------------------------------- the fused whole-model kernel
// One launch = one decode step for all layers (paper abstract, Section 3).  Phases per layer, each
// followed by a grid barrier: [RMSNorm + QKV projection + RoPE + cache append] [split-KV attention
// + merge] [output projection + residual] [RMSNorm + gate/up projection + SwiGLU] [down projection
// + residual]; then the final norm and LM head.
template <int WD, int B>
__global__ void __launch_bounds__(kThreads) fused_decode_kernel(DevModel M, DevKV KV, const int* __restrict__ tokens,
                                                                const int* __restrict__ pos, float* __restrict__ logits,
                                                                int batch, u32 bar_base) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    if (!inputs_ok(M, KV, tokens, pos, batch)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicExch(M.status, kStatusRange);
        return;
    }
    typedef CoherentIO IO;
    u32 gen = bar_base;
    // residual stream starts as the embedding rows; per-(sequence, kv head) arrival counters to 0
    {
        const int tot = batch * M.d;
        for (int i = blockIdx.x * kThreads + threadIdx.x; i < tot; i += gridDim.x * kThreads) {
            int b = i / M.d, c = i % M.d;
            IO::st(M.x + (size_t)b * M.d + c, bf_to_f(M.embed[(size_t)tokens[b] * M.d + c]));
        }
        if (blockIdx.x == 0 && threadIdx.x < batch * M.Hkv) xst_u32(&M.head_ctr[threadIdx.x], 0u);
    }
    for (int l = 0; l < M.L; l++) {
        const PLayer& Ly = M.layers[l];
        {
            ActSrc src = l == 0 ? ActSrc{M.embed, tokens, 0, Ly.g1, M.eps} : ActSrc{M.x, nullptr, (size_t)M.d, Ly.g1, M.eps};
            EpiQKV<IO> epi{M, KV, pos, l};
            gemv_phase<WD, B, IO>(Ly.qkv, src, batch, lds, epi);
        }
        if (!grid_barrier(M, ++gen)) return;
        attention_phase<IO>(M, KV, pos, batch, l, lds, true);
        if (!grid_barrier(M, ++gen)) return;
        {
            ActSrc src{M.attn_o, nullptr, (size_t)M.Hq * M.hd, nullptr, 0.f};
            EpiResidual<IO> epi{M.x, M.d};
            gemv_phase<WD, B, IO>(Ly.o, src, batch, lds, epi);
        }
        if (!grid_barrier(M, ++gen)) return;
        {
            ActSrc src{M.x, nullptr, (size_t)M.d, Ly.g2, M.eps};
            EpiSwiGLU<IO> epi{M.h, M.F};
            gemv_phase<WD, B, IO>(Ly.gu, src, batch, lds, epi);
        }
        if (!grid_barrier(M, ++gen)) return;
        {
            ActSrc src{M.h, nullptr, (size_t)M.F, nullptr, 0.f};
            EpiResidual<IO> epi{M.x, M.d};
            gemv_phase<WD, B, IO>(Ly.down, src, batch, lds, epi);
        }
        if (!grid_barrier(M, ++gen)) return;
    }
    {
        ActSrc src{M.x, nullptr, (size_t)M.d, M.gf, M.eps};
        EpiStore epi{logits, M.V};
        if (M.lm.wd == WD) gemv_phase<WD, B, IO>(M.lm, src, batch, lds, epi);
        else gemv_phase<W_BF16, B, IO>(M.lm, src, batch, lds, epi);
    }
}
constexpr int kBarriersPerLayer = 5;

// ---------------------------------------------------------------- per-operation baseline kernels
__global__ void __launch_bounds__(kThreads) op_embed(DevModel M, DevKV KV, const int* tokens, const int* pos, int batch) {
    if (!inputs_ok(M, KV, tokens, pos, batch)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicExch(M.status, kStatusRange);
        return;
    }
    const int tot = batch * M.d;
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < tot; i += gridDim.x * kThreads) {
        int b = i / M.d, c = i % M.d;
        M.x[(size_t)b * M.d + c] = bf_to_f(M.embed[(size_t)tokens[b] * M.d + c]);
    }
}
// grid = batch
__global__ void __launch_bounds__(kThreads) op_rmsnorm(const float* x, const bf16_t* gain, float* out, int d, float eps) {
    __shared__ float red[kWaves];
    const float* xr = x + (size_t)blockIdx.x * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += kThreads) ss += xr[i] * xr[i];
    float r = 1.0f / sqrtf(block_sum(ss, red) / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += kThreads) out[(size_t)blockIdx.x * d + i] = xr[i] * bf_to_f(gain[i]) * r;
}
enum { EPI_STORE = 0, EPI_RESIDUAL = 1 };
template <int WD, int B>
__global__ void __launch_bounds__(kThreads) op_gemv(PMat W, const float* in, int in_stride, float* out, int batch, int epi_kind) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    ActSrc src{in, nullptr, (size_t)in_stride, nullptr, 0.f};
    if (epi_kind == EPI_RESIDUAL) {
        EpiResidual<PlainIO> epi{out, W.n};
        gemv_phase<WD, B, PlainIO>(W, src, batch, lds, epi);
    } else {
        EpiStore epi{out, W.n};
        gemv_phase<WD, B, PlainIO>(W, src, batch, lds, epi);
    }
}
// y holds raw QKV outputs in packed row order [B][rows]
__global__ void __launch_bounds__(kThreads) op_rope_append(DevModel M, DevKV KV, const int* tokens, const int* pos, int batch, int layer) {
    if (!inputs_ok(M, KV, tokens, pos, batch)) return;
    const int rows = (M.Hq + 2 * M.Hkv) * M.hd, npairs = rows / 2;
    EpiQKV<PlainIO> epi{M, KV, pos, layer};
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < npairs * batch; i += gridDim.x * kThreads) {
        int b = i / npairs, p = i % npairs;
        const float* y = M.y + (size_t)b * rows + 2 * p;
        epi(p, b, y[0], y[1]);
    }
}
__global__ void __launch_bounds__(kThreads) op_attn_partial(DevModel M, DevKV KV, const int* tokens, const int* pos, int batch, int layer) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    if (!inputs_ok(M, KV, tokens, pos, batch)) return;
    attention_phase<PlainIO>(M, KV, pos, batch, layer, lds, false);
}
// grid = batch * Hkv; must be launched with the same share (= partial grid / (batch*Hkv)) in `share`
__global__ void __launch_bounds__(kThreads) op_attn_merge(DevModel M, DevKV KV, const int* tokens, const int* pos, int batch, int share) {
    if (!inputs_ok(M, KV, tokens, pos, batch)) return;
    int b = blockIdx.x / M.Hkv, j = blockIdx.x % M.Hkv;
    int ns = attn_nsplit(pos[b], share);
    const int G = M.Hq / M.Hkv;
    if (M.hd == 64 && G == 4) attn_merge<64, 4, PlainIO>(M, b, j, ns);
    else if (M.hd == 128 && G == 4) attn_merge<128, 4, PlainIO>(M, b, j, ns);
    else if (M.hd == 128 && G == 8) attn_merge<128, 8, PlainIO>(M, b, j, ns);
}
// y holds raw gate/up outputs, rows interleaved [B][2F]
__global__ void __launch_bounds__(kThreads) op_swiglu(DevModel M, int batch) {
    EpiSwiGLU<PlainIO> epi{M.h, M.F};
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < M.F * batch; i += gridDim.x * kThreads) {
        int b = i / M.F, p = i % M.F;
        const float* y = M.y + (size_t)b * 2 * M.F + 2 * p;
        epi(p, b, y[0], y[1]);
    }
}

// ---------------------------------------------------------------- loaders and utilities
enum { REPACK_COPY = 0, REPACK_ROPE = 1, REPACK_INTERLEAVE = 2 };
// dst row r  <-  source row per mode.  row_bytes is a multiple of 2.
__global__ void __launch_bounds__(kThreads) k_repack_rows(uint8_t* dst, const uint8_t* src_a, const uint8_t* src_b, int n_rows,
                                                         size_t row_bytes, int mode, int hd) {
    for (int r = blockIdx.x; r < n_rows; r += gridDim.x) {
        const uint8_t* src;
        if (mode == REPACK_ROPE) {
            int head = r / hd, within = r % hd;
            src = src_a + (size_t)(head * hd + within / 2 + (within & 1) * (hd / 2)) * row_bytes;
        } else if (mode == REPACK_INTERLEAVE) {
            src = ((r & 1) ? src_b : src_a) + (size_t)(r / 2) * row_bytes;
        } else {
            src = src_a + (size_t)r * row_bytes;
        }
        uint8_t* d = dst + (size_t)r * row_bytes;
        if (row_bytes % 16 == 0) {
            for (size_t i = threadIdx.x; i < row_bytes / 16; i += kThreads) ((u32x4*)d)[i] = ((const u32x4*)src)[i];
        } else {
            for (size_t i = threadIdx.x; i < row_bytes / 2; i += kThreads) ((uint16_t*)d)[i] = ((const uint16_t*)src)[i];
        }
    }
}
__global__ void k_rope_table(float2* rope, int max_ctx, int hd, double theta) {
    int half = hd / 2;
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= max_ctx * half) return;
    int p = i / half, f = i % half;
    double ang = (double)p * pow(theta, -2.0 * (double)f / (double)hd);
    double s, c;
    sincos(ang, &s, &c);
    rope[i] = make_float2((float)c, (float)s);
}
// canonical [n][Hkv][hd] rows <-> cache planes; dir 0 = fill cache, 1 = read cache
__global__ void k_kv_copy(DevKV KV, int L_unused, int Hkv, int hd, bf16_t* plane_base_k, bf16_t* plane_base_v, size_t plane_stride_j,
                          int pos0, int n, bf16_t* k_can, bf16_t* v_can, int dir) {
    size_t tot = (size_t)n * Hkv * hd;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < tot; i += (size_t)gridDim.x * blockDim.x) {
        int e = i % hd, j = (i / hd) % Hkv, t = i / ((size_t)hd * Hkv);
        size_t off = (size_t)j * plane_stride_j + (size_t)(pos0 + t) * hd + e;
        if (dir == 0) { plane_base_k[off] = k_can[i]; plane_base_v[off] = v_can[i]; }
        else { k_can[i] = plane_base_k[off]; v_can[i] = plane_base_v[off]; }
    }
}
// Dequantise packed matrix element-wise into canonical [N][K] fp32.  map: 0 identity, 1 RoPE-pair
// block, 2 interleave (even rows: parity 0, odd rows: parity 1); row_off = first packed row.
__global__ void k_dequant(PMat W, float* out, int n_can, int map, int parity, int row_off, int hd) {
    size_t tot = (size_t)n_can * W.k;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < tot; i += (size_t)gridDim.x * blockDim.x) {
        int r = i / W.k, c = i % W.k;
        int pr;
        if (map == 1) { int head = r / hd, within = r % hd, half = hd / 2; pr = head * hd + 2 * (within % half) + within / half; }
        else if (map == 2) pr = 2 * r + parity;
        else pr = r;
        pr += row_off;
        const uint8_t* row = W.w + (size_t)pr * W.row_bytes();
        float v;
        if (W.wd == W_BF16) v = bf_to_f(((const bf16_t*)row)[c]);
        else if (W.wd == W_INT8) v = (float)(int)((const int8_t*)row)[c] * f16_to_f(W.s[pr]);
        else {
            int ng = W.k / 128;
            uint8_t byte = row[c >> 1];
            int code = (c & 1) ? (byte >> 4) : (byte & 15);
            v = ((float)code - f16_to_f(W.z[(size_t)pr * ng + c / 128])) * f16_to_f(W.s[(size_t)pr * ng + c / 128]);
        }
        out[i] = v;
    }
}
__global__ void k_fill_u32(u32* p, size_t n, u32 v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

}  // namespace ff
