// Device-side structures and primitives shared by the fused whole-model kernel and the
// per-operation baseline kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ff {

typedef unsigned int u32;
typedef unsigned long long u64;
typedef __attribute__((ext_vector_type(4))) u32 u32x4;
typedef __attribute__((ext_vector_type(2))) u32 u32x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef uint16_t bf16_t;   // raw bits
typedef uint16_t f16_t;    // raw bits

constexpr int kThreads = 256;            // threads per workgroup (4 waves, one per SIMD)
constexpr int kWaves = kThreads / 64;
constexpr int kMaxBatch = 4;        // sequences one pass of the row-partitioned paths works on
constexpr int kMaxBatchFused = 8;   // sequences the regular RoPE / position / mailbox regions of the fused kernel's LDS are laid out for
constexpr int kMaxBatchWide = 16;   // sequences of a wide pass (bf16 weights, see ff_wide.h)
constexpr int kMaxBatchApi = 16;    // sequences one decode step accepts (one wide pass, or passes of kMaxBatch)
constexpr int kMaxSplits = 64;           // max KV splits per (sequence, kv head)
#ifndef FF_MIN_SPLIT
#define FF_MIN_SPLIT 64   // can be overridden at build time for sweeps (32 and 128 both measured 2 % slower at ctx 1024)
#endif
constexpr int kMinSplitLen = FF_MIN_SPLIT;   // do not split the cache finer than this many rows
constexpr int kLdsActBytes = 128 * 1024; // LDS region holding the staged activation vector(s)
constexpr int kLdsAuxBytes = 24 * 1024;  // partial sums of earlier K segments (per wave), then kLdsXsumBytes of per-unit input sums
constexpr int kLdsXsumBytes = 4 * 1024;  // tail of the aux region: sum of every staged 32-element unit (int4 matrix-core path)
constexpr int kLdsRopeBytes = 8 * 64 * 8;   // behind the aux region: (cos, sin) rows of up to 8 sequences
constexpr int kLdsMiscBytes = 256;          // then: reduction scratch, positions, vote slots
constexpr int kLdsPairBytes = 1024;         // then: mailboxes of wave pairs that share a row group (gemv_run_quad)
constexpr int kLdsFusedBytes = kLdsActBytes + kLdsAuxBytes + kLdsRopeBytes + kLdsMiscBytes + kLdsPairBytes;
constexpr int kSpinLimit = 1 << 16;


enum { W_BF16 = 0, W_INT8 = 1, W_INT4 = 2 };

// A projection matrix in packed (device-private) row order.
struct PMat {
    const uint8_t* w;   // rows of row_bytes each
    const f16_t* s;     // int8: [n]; int4: [n][k/128]
    const f16_t* z;     // int4: [n][k/128]
    int n, k;           // rows (outputs), columns (inputs)
    int wd;
    __host__ __device__ size_t row_bytes() const { return wd == W_BF16 ? (size_t)k * 2 : wd == W_INT8 ? (size_t)k : (size_t)k / 2; }
};
#define FF_PMAT_FIELDS(p) PMat{(p).w, (p).s, (p).z, (p).n, (p).k, (p).wd}

struct PLayer {
    const bf16_t* g1;   // attention pre-norm gain
    const bf16_t* g2;   // FFN pre-norm gain
    PMat qkv;           // rows: q heads, k heads (RoPE partners adjacent), then v heads
    PMat o;
    PMat gu;            // rows 2i = gate_i, 2i+1 = up_i
    PMat down;
};

// Order of the gate/up row pairs in the packed copy.  Identity (nw == 0): packed pair q = FFN unit q.
// Interleaved (nw = waves in the grid, P = F / nw pairs per wave): the wave that owns packed pairs
// [w P, (w + 1) P) holds FFN units w, w + nw, w + 2 nw, ... so that the i-th pair of EVERY wave
// together cover the contiguous units [i nw, (i + 1) nw): a K chunk of the down projection's input is
// complete as soon as every wave has finished a fixed, small number of its pairs (see glu_run).
struct GuPerm {
    int P, nw;
    __host__ __device__ int unit_of_pair(int q) const { return nw ? (q % P) * nw + q / P : q; }
    __host__ __device__ int pair_of_unit(int f) const { return nw ? (f % nw) * P + f / nw : f; }
};

// Everything the kernels need about the model and its exchange buffers.
struct DevModel {
    int L, d, Hq, Hkv, hd, F, V;
    GuPerm gu;               // gate/up pair order of the packed copy
    float eps;
    const PLayer* layers;    // device array [L]
    const bf16_t* embed;
    const bf16_t* gf;
    PMat lm;
    // exchange buffers (device scratch)
    // plain exchange buffers (per-operation kernels)
    float* x;        // residual stream            [B][d]
    float* xn;       // normed activation (per-op)  [B][d]
    float* q;        // rotated queries            [B][Hq*hd]
    float* kvcur;    // this step's k,v (bf16-rounded values as fp32) [B][2][Hkv*hd]
    float* attn_o;   // merged attention output    [B][Hq*hd]
    float* h;        // SwiGLU output              [B][F]
    float* y;        // per-op: raw projection out [B][max rows]
    float* part_m;   // split partials             [B][Hq][kMaxSplits]
    float* part_l;
    float* part_o;   //                            [B][Hq][kMaxSplits][hd]
    // tagged exchange buffers of the fused kernel: (fp32 bits, tag) pairs, same shapes as above
    u32x2* tq;  u32x2* tkvcur;
    // the vectors every workgroup reads whole, in the compact 4-byte format (value with a 2-bit write
    // counter in its lowest mantissa bits): residual stream (two buffers), sublayer output, merged
    // attention output, SwiGLU output
    u32* cx;  u32* cx2;  u32* cdelta;  u32* cattn_o;  u32* ch;
    // wide pass (ff_wide.h): residual rows [16][d] (each row touched by its owning workgroup only), images of
    // the consumers' LDS layout for the d-wide inputs, the merged attention output and the SwiGLU output, the
    // workgroups' partial sums of squares [workgroups][16], one epoch word per workgroup
    float* wxres;  uint8_t* wimg_x;  uint8_t* wimg_a;  uint8_t* wimg_h;  float* wsspart;  u32* wflag;  float* wxch;  u32* wpflag;
    u32* stepctr;    // [0] fused launches executed so far on these buffers (skipped steps do not count); [1] sequences the last one served
    u32x2* tpart_m;  u32x2* tpart_l;  u32x2* tpart_o;
    int* status;
    u64* dbg;        // optional timeline buffer (null unless enabled through the debug entry point)
};

struct DevKV {
    bf16_t* base;        // [L][batch][Hkv][2][max_ctx][hd]
    const float2* rope;  // [max_ctx][hd/2] (cos, sin)
    int max_ctx, batch;
    int seq0;            // first sequence of the current pass (kernels number their sequences from 0)
    int step_batch;      // sequences of the whole decode step (all passes)
    __device__ bf16_t* plane(const DevModel& M, int l, int b, int j, int kv) const {
        return base + ((((size_t)l * batch + (seq0 + b)) * M.Hkv + j) * 2 + kv) * (size_t)max_ctx * M.hd;
    }
};

// Pointers that reach a kernel inside structures read from memory lose their address space; a
// generic-address (FLAT) access counts against the LDS counter as well as the vector-memory one and
// forces full waits.  Everything dereferenced in device code goes through these casts.
#define FF_GLOBAL __attribute__((address_space(1)))
template <class T> __device__ __forceinline__ const FF_GLOBAL T* as_global(const T* p) { return (const FF_GLOBAL T*)p; }
template <class T> __device__ __forceinline__ FF_GLOBAL T* as_global(T* p) { return (FF_GLOBAL T*)p; }
// Read-only data that no kernel writes (the layer descriptors): uniform loads through the constant
// address space are scalar loads, which do not queue behind the wave's vector loads and stores.
#define FF_CONST __attribute__((address_space(4)))
template <class T> __device__ __forceinline__ const FF_CONST T* as_const(const T* p) { return (const FF_CONST T*)p; }

// ---------------------------------------------------------------- coherent exchange accesses
// Activations exchanged between workgroups inside one launch must bypass the per-XCD L2's
// non-coherent lines (an agent-scope acquire or release fence costs several microseconds on this
// chip): they are written with agent-scope relaxed atomic stores (write through to the coherence
// point) and read with agent-scope relaxed atomic loads of at most 8 bytes (see the tagged
// exchange format).  Buffer loads with the matching cache-policy bit are not used: they were
// observed to keep returning a stale copy while polling.
__device__ __forceinline__ void xst(float* p, float v) {
    __hip_atomic_store(as_global((u32*)p), __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void xst2(float* p, float a, float b) {
    u64 v = (u64)__float_as_uint(a) | ((u64)__float_as_uint(b) << 32);
    __hip_atomic_store(as_global((u64*)p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u32 xld_u32(const u32* p) { return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void xst_u32(u32* p, u32 v) { __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ u32 xadd_u32(u32* p, u32 v) { return __hip_atomic_fetch_add(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

struct PlainIO {   // launch-boundary ordered accesses (per-operation kernels)
    static __device__ __forceinline__ float ld(const float* base, int i) { return as_global(base)[i]; }
    static __device__ __forceinline__ float2 ld2(const float* base, int i) {
        f32x2 v = *as_global((const f32x2*)(base + i));
        return make_float2(v.x, v.y);
    }
    static __device__ __forceinline__ float4 ld4(const float* base, int i) {
        f32x4 v = *as_global((const f32x4*)(base + i));
        return make_float4(v.x, v.y, v.z, v.w);
    }
    static __device__ __forceinline__ void st(float* p, float v) { *as_global(p) = v; }
    static __device__ __forceinline__ void st2(float* p, float a, float b) { *as_global((f32x2*)p) = f32x2{a, b}; }
    static __device__ __forceinline__ void st4(float* p, float4 v) { *as_global((f32x4*)p) = f32x4{v.x, v.y, v.z, v.w}; }
};
// ---------------------------------------------------------------- scalar helpers
__device__ __forceinline__ float bf_lo(u32 w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(u32 w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ float bf_to_f(bf16_t h) { return __uint_as_float((u32)h << 16); }
// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ bf16_t f_to_bf(float f) {
    u32 u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float f16_to_f(f16_t h) {
    _Float16 v;
    __builtin_memcpy(&v, &h, 2);
    return (float)v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ u32x4 ldg_stream(const void* p) { return __builtin_nontemporal_load(as_global((const u32x4*)p)); }

// A sequence whose token is kTokenSkip takes no part in the step (it has stopped while the rest of
// the batch decodes on): its position is ignored, its cache and its logits row are left as they are.
// Inside the kernels such a sequence has position -1; it is carried through the layers as a
// placeholder (token 0 at an empty cache) whose k, v and logits are never stored, so the launch
// shape and the exchange protocol do not depend on which sequences are active.
constexpr int kTokenSkip = -1;
__device__ __forceinline__ int step_pos(const int* tokens, const int* pos, int b) { return tokens[b] == kTokenSkip ? -1 : pos[b]; }

}  // namespace ff
