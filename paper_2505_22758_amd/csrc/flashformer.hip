// C ABI of the MI355X whole-model decode library (see include/flashformer.h).
#include "../../include/flashformer.h"
#include "ff_fused.h"
#include "ff_ops.h"
#include "ff_stack.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace ff;

// Exchange scratch of ff_decode_step_static: one copy per GPU the library runs on, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels receive
// the device address obtained from it (static_scratch_ptr below).
constexpr size_t kStaticScratchBytes = FF_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static __device__ unsigned int sink_word;   // never-written target that keeps k_stream_read's loads alive

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}
#define HIPCHK(expr)                                                                                   \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess) return fail(FF_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));  \
    } while (0)

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct MatPlan { size_t w, s, z; int n, k, wd; };   // byte offsets into packed_dev
struct LayerPlan { size_t g1, g2; MatPlan qkv, o, gu, down; };
struct Plan {
    size_t layers_tab;
    std::vector<LayerPlan> layers;
    size_t embed, gf;
    MatPlan lm;
    size_t packed_bytes;
    // scratch
    size_t x, xn, q, kvcur, attn_o, h, y, part_m, part_l, part_o, status, scratch_bytes;
    size_t cx, cx2, cdelta, tq, tkvcur, cattn_o, ch, stepctr, tpart_m, tpart_l, tpart_o;
    size_t wxres, wimg_x, wimg_a, wimg_h, wsspart, wflag, wxch, wpflag;   // wide pass only (zero bytes otherwise)
};

size_t mat_w_bytes(int n, int k, int wd) { return wd == W_BF16 ? (size_t)n * k * 2 : wd == W_INT8 ? (size_t)n * k : (size_t)n * k / 2; }
size_t mat_s_bytes(int n, int k, int wd) { return wd == W_INT8 ? (size_t)n * 2 : wd == W_INT4 ? (size_t)n * (k / 128) * 2 : 0; }

MatPlan plan_mat(size_t& off, int n, int k, int wd) {
    MatPlan p{0, 0, 0, n, k, wd};
    p.w = off; off = align256(off + mat_w_bytes(n, k, wd));
    p.s = off; off = align256(off + mat_s_bytes(n, k, wd));
    p.z = off; off = align256(off + (wd == W_INT4 ? mat_s_bytes(n, k, wd) : 0));
    return p;
}

int check_config(const ff_config* c) {
    if (!c) return fail(FF_ERR_ARG, "config is null");
    if (c->n_layers < 1 || c->d_model < 8 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 8 || c->vocab < 2)
        return fail(FF_ERR_ARG, "non-positive model dimension");
    if (c->max_batch < 1 || c->max_batch > kMaxBatchApi) return fail(FF_ERR_ARG, "max_batch %d outside [1,%d]", c->max_batch, kMaxBatchApi);
    if (c->wdtype < 0 || c->wdtype > 2) return fail(FF_ERR_ARG, "unknown wdtype %d", c->wdtype);
    if (c->n_q_heads % c->n_kv_heads) return fail(FF_ERR_UNSUPPORTED, "n_q_heads must be a multiple of n_kv_heads");
    int G = c->n_q_heads / c->n_kv_heads;
    bool inst = (c->head_dim == 64 && G == 4) || (c->head_dim == 128 && G == 4) || (c->head_dim == 128 && G == 8);
    if (!inst) return fail(FF_ERR_UNSUPPORTED, "no attention instance for head_dim %d with %d query heads per kv head", c->head_dim, G);
    int epu = c->wdtype == W_BF16 ? 8 : c->wdtype == W_INT8 ? 16 : 128;
    int qd = c->n_q_heads * c->head_dim;
    if (c->d_model % epu || qd % epu || c->d_ffn % epu)
        return fail(FF_ERR_UNSUPPORTED, "d_model, n_q_heads*head_dim and d_ffn must be multiples of %d for this weight type", epu);
    if (c->d_model % 8 || c->d_ffn % 2 || c->vocab < 2) return fail(FF_ERR_UNSUPPORTED, "d_model must be a multiple of 8");
    // the row partition among waves is computed in 32 bits: (rows / 2) * (waves in the grid) < 2^32
    if (c->vocab > (1 << 21) || c->d_ffn > (1 << 20) || c->d_model > (1 << 20) || qd > (1 << 20))
        return fail(FF_ERR_UNSUPPORTED, "matrix with more than 2^21 rows");
    // with two or more sequences per pass (matrix-core projections) a row is normalised in a
    // single staging pass (8 quads per thread)
    if (c->max_batch > 1 && c->d_model > 8192)
        return fail(FF_ERR_UNSUPPORTED, "d_model %d > 8192 with max_batch > 1 is not supported", c->d_model);
    if ((size_t)c->d_model * 4 * std::min(c->max_batch, kMaxBatch) > (size_t)kLdsActBytes)
        return fail(FF_ERR_UNSUPPORTED, "d_model %d x max_batch %d does not fit the on-chip input buffer (RMSNorm needs the whole row)", c->d_model, c->max_batch);
    return FF_OK;
}

// The wide instance gives every workgroup a contiguous range of rows of each projection, in tiles
// of 16 whose accumulators stay in registers: at most kDenseMaxTiles tiles per workgroup (on a grid
// of n_cta workgroups), and whole groups of four rows of the d-wide projections.
bool wide_fits(const ff_config& c, int n_cta) {
    const int qkv_rows = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    const int rows = std::max(std::max(qkv_rows, c.d_model), 2 * c.d_ffn);
    const int groups = ((rows + 3) / 4 + n_cta - 1) / n_cta;
    return (4 * groups + 15) / 16 <= kDenseMaxTiles && c.d_model % 8 == 0 && qkv_rows % 4 == 0;
}
constexpr int kGridCtas = 256;   // workgroups of the fused kernel's grid on the chip the kernels are built for

// Sequences one pass of the fused kernel serves: up to 4 on the row-partitioned paths (paper Section
// 5.2), or, with bf16 or int8 weights and a model created for more than that, up to 16 in one wide
// pass.
// FF_WIDE_MIN (experiments): smallest batch that takes the wide pass (default 5; it measured equal
// to the former eight-sequence instance at 5 sequences and faster from 6 on, slower than the
// four-sequence path below that).
int wide_min_batch() {
    const char* e = getenv("FF_WIDE_MIN");
    const int v = e ? atoi(e) : 0;
    return v > 0 ? v : kMaxBatch + 1;
}
int fused_pass_rows(const ff_config& c) {
    // (quantised layers with a bf16 LM head keep the passes of four: the wide pass runs the LM head inside the kernel, in the layers' format)
    // (int4: the wide pass takes a row's scales and zeros four groups at a time: every input width a multiple of 512)
    const bool k512 = c.d_model % 512 == 0 && (c.n_q_heads * c.head_dim) % 512 == 0 && c.d_ffn % 512 == 0;
    const bool fmt_ok = c.wdtype == W_BF16 || ((c.wdtype == W_INT8 || (c.wdtype == W_INT4 && k512)) && c.quant_lm_head);
    if (fmt_ok && c.max_batch >= wide_min_batch() && wide_fits(c, kGridCtas)) return kMaxBatchWide;
    return std::min(c.max_batch, kMaxBatch);
}
// Does a pass of `batch` sequences (batch <= fused_pass_rows) run on the wide instance?  A model created
// for more than four sequences has the wide pass's buffers; with int8 weights its passes of four take the
// wide instance too (8B shape, context 4096: 3.53 ms against 3.87 ms on the row-partitioned path; at
// three sequences the two are equal, below that and with bf16 weights the row-partitioned path is faster).
bool pass_is_wide(const ff_config& c, int batch) {
    const bool env = getenv("FF_WIDE_MIN") != nullptr;
    return fused_pass_rows(c) == kMaxBatchWide && batch >= (!env && c.wdtype == W_INT8 ? kMaxBatch : wide_min_batch());
}

Plan make_plan(const ff_config& c) {
    Plan P;
    size_t off = 0;
    P.layers_tab = off; off = align256(off + sizeof(PLayer) * c.n_layers);
    int qkv_rows = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, qd = c.n_q_heads * c.head_dim;
    for (int l = 0; l < c.n_layers; l++) {
        LayerPlan L;
        L.g1 = off; off = align256(off + (size_t)c.d_model * 2);
        L.g2 = off; off = align256(off + (size_t)c.d_model * 2);
        L.qkv = plan_mat(off, qkv_rows, c.d_model, c.wdtype);
        L.o = plan_mat(off, c.d_model, qd, c.wdtype);
        L.gu = plan_mat(off, 2 * c.d_ffn, c.d_model, c.wdtype);
        L.down = plan_mat(off, c.d_model, c.d_ffn, c.wdtype);
        P.layers.push_back(L);
    }
    P.embed = off; off = align256(off + (size_t)c.vocab * c.d_model * 2);
    P.gf = off; off = align256(off + (size_t)c.d_model * 2);
    P.lm = plan_mat(off, c.vocab, c.d_model, c.quant_lm_head ? c.wdtype : W_BF16);
    P.packed_bytes = off;

    size_t s = 0;
    size_t mb = fused_pass_rows(c);   // exchange buffers hold one pass
    auto take = [&](size_t bytes) { size_t o = s; s = align256(s + bytes); return o; };
    P.x = take(mb * c.d_model * 4);
    P.xn = take(mb * c.d_model * 4);
    P.q = take(mb * qd * 4);
    P.kvcur = take(mb * 2 * c.n_kv_heads * c.head_dim * 4);
    P.attn_o = take(mb * qd * 4);
    P.h = take(mb * c.d_ffn * 4);
    size_t ymax = std::max((size_t)qkv_rows, (size_t)2 * c.d_ffn);
    P.y = take(mb * ymax * 4);
    P.part_m = take(mb * c.n_q_heads * kMaxSplits * 4);
    P.part_l = take(mb * c.n_q_heads * kMaxSplits * 4);
    P.part_o = take(mb * c.n_q_heads * kMaxSplits * c.head_dim * 4);
    P.cx = take(mb * c.d_model * 4);
    P.cx2 = take(mb * c.d_model * 4);
    P.cdelta = take(mb * c.d_model * 4);
    P.tq = take(mb * qd * 8);
    P.tkvcur = take(mb * 2 * c.n_kv_heads * c.head_dim * 8);
    P.cattn_o = take(mb * qd * 4);
    P.ch = take(mb * c.d_ffn * 4);
    P.stepctr = take(256);
    P.tpart_m = take(mb * c.n_q_heads * kMaxSplits * 8);
    P.tpart_l = take(mb * c.n_q_heads * kMaxSplits * 8);
    P.tpart_o = take(mb * c.n_q_heads * kMaxSplits * c.head_dim * 8);
    const bool wide = mb == (size_t)kMaxBatchWide;
    P.wxres = take(wide ? mb * c.d_model * 4 : 0);
    P.wimg_x = take(wide ? wide_img_bytes(c.d_model) : 0);
    P.wimg_a = take(wide ? wide_img_bytes(qd) : 0);
    P.wimg_h = take(wide ? wide_img_bytes(c.d_ffn) : 0);
    P.wsspart = take(wide ? (size_t)kGridCtas * kMaxBatchWide * 4 : 0);
    P.wflag = take(wide ? (size_t)kGridCtas * 4 : 0);
    P.wxch = take(wide ? (size_t)kGridCtas * kWideXchFloats * 4 : 0);   // partial sums handed to the partner workgroup (K-split projections)
    P.wpflag = take(wide ? (size_t)kGridCtas * 4 : 0);
    P.status = take(256);
    P.scratch_bytes = s;
    return P;
}

}  // namespace

struct ff_model {
    ff_config cfg;
    Plan plan;
    uint8_t* packed;
    uint8_t* scratch;
    DevModel dev;
    std::vector<PLayer> host_layers;
    std::vector<char> layer_loaded;
    bool head_loaded;
    int n_cta;
    size_t lds_bytes;
    int mute_wg = -1;   // test hook (ff_debug_mute_workgroup)
    int switches = 0;   // kSw* bits of the fused launches (ff_debug_set_overlap, ff_debug_set_attention_balance)
    int glu_off = -1;   // >= 0: LDS offset of the staged SwiGLU output when gate/up + down run as one stream (glu_run)
};
struct ff_kv {
    ff_model* model;
    DevKV dev;
    int batch, max_ctx;
};

namespace {

PMat to_pmat(const MatPlan& p, uint8_t* base) {
    PMat m;
    m.w = base + p.w;
    m.s = (const f16_t*)(base + p.s);
    m.z = (const f16_t*)(base + p.z);
    m.n = p.n; m.k = p.k; m.wd = p.wd;
    return m;
}

// copy canonical rows [n_rows] of `src` into packed rows starting at dst_row, with row mapping
int repack(const MatPlan& dst, uint8_t* packed, int dst_row, int n_rows, const ff_matrix& a, const ff_matrix* b, int mode, int hd,
           const GuPerm& perm, hipStream_t st) {
    if (!a.w || (b && !b->w)) return fail(FF_ERR_ARG, "matrix pointer is null");
    size_t rb = dst.wd == W_BF16 ? (size_t)dst.k * 2 : dst.wd == W_INT8 ? (size_t)dst.k : (size_t)dst.k / 2;
    int grid = std::min(n_rows, 4096);
    k_repack_rows<<<grid, kThreads, 0, st>>>(packed + dst.w + (size_t)dst_row * rb, (const uint8_t*)a.w, b ? (const uint8_t*)b->w : nullptr,
                                             n_rows, rb, mode, hd, perm);
    if (dst.wd != W_BF16) {
        if (!a.s || (b && !b->s)) return fail(FF_ERR_ARG, "scale pointer is null for a quantised matrix");
        size_t sb = dst.wd == W_INT8 ? 2 : (size_t)(dst.k / 128) * 2;
        k_repack_rows<<<grid, kThreads, 0, st>>>(packed + dst.s + (size_t)dst_row * sb, (const uint8_t*)a.s, b ? (const uint8_t*)b->s : nullptr,
                                                 n_rows, sb, mode, hd, perm);
        if (dst.wd == W_INT4) {
            if (!a.z || (b && !b->z)) return fail(FF_ERR_ARG, "zero-point pointer is null for an int4 matrix");
            k_repack_rows<<<grid, kThreads, 0, st>>>(packed + dst.z + (size_t)dst_row * sb, (const uint8_t*)a.z,
                                                     b ? (const uint8_t*)b->z : nullptr, n_rows, sb, mode, hd, perm);
        }
    }
    HIPCHK(hipGetLastError());
    return FF_OK;
}

template <typename K>
int set_lds(K kernel, size_t bytes) {
    HIPCHK(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    return FF_OK;
}

int check_step_args(ff_model* m, const int32_t* tokens, const int32_t* pos, ff_kv* kv, float* logits, int32_t batch) {
    if (!m || !tokens || !pos || !kv || !logits) return fail(FF_ERR_ARG, "null argument to decode step");
    if (kv->model != m) return fail(FF_ERR_ARG, "kv cache belongs to a different model");
    if (batch < 1 || batch > m->cfg.max_batch || batch > kv->batch)
        return fail(FF_ERR_ARG, "batch %d outside [1, min(max_batch %d, cache batch %d)]", batch, m->cfg.max_batch, kv->batch);
    for (int l = 0; l < m->cfg.n_layers; l++)
        if (!m->layer_loaded[l]) return fail(FF_ERR_ARG, "layer %d has not been loaded", l);
    if (!m->head_loaded) return fail(FF_ERR_ARG, "embedding / LM head have not been loaded");
    return FF_OK;
}

template <int WD, int B>
int launch_gemv(ff_model* m, const PMat& W, const float* in, int in_stride, float* out, int batch, int epi, hipStream_t st, const int* skip_tokens = nullptr) {
    auto kern = op_gemv<WD, B>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] { attr_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)m->lds_bytes); });
    if (attr_err != hipSuccess) return fail(FF_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(attr_err));
    kern<<<m->n_cta, kThreads, m->lds_bytes, st>>>(W, in, in_stride, out, batch, epi, skip_tokens);
    return FF_OK;
}
template <int B>
int gemv_any(ff_model* m, const PMat& W, const float* in, int in_stride, float* out, int batch, int epi, hipStream_t st, const int* skip_tokens) {
    switch (W.wd) {
        case W_BF16: return launch_gemv<W_BF16, B>(m, W, in, in_stride, out, batch, epi, st, skip_tokens);
        case W_INT8: return launch_gemv<W_INT8, B>(m, W, in, in_stride, out, batch, epi, st, skip_tokens);
        default: return launch_gemv<W_INT4, B>(m, W, in, in_stride, out, batch, epi, st, skip_tokens);
    }
}
// skip_tokens (EPI_STORE only, may be null): the tokens of the `batch` sequences; rows of sequences that sit the step out are not written
int gemv_op(ff_model* m, const PMat& W, const float* in, int in_stride, float* out, int batch, int epi, hipStream_t st, const int* skip_tokens = nullptr) {
    if (batch == 1) return gemv_any<1>(m, W, in, in_stride, out, batch, epi, st, skip_tokens);
    if (batch == 2) return gemv_any<2>(m, W, in, in_stride, out, batch, epi, st, skip_tokens);
    return gemv_any<4>(m, W, in, in_stride, out, batch, epi, st, skip_tokens);
}

}  // namespace

extern "C" {

const char* ff_last_error(void) { return g_err.c_str(); }

int ff_model_bytes(const ff_config* cfg, size_t* packed_bytes, size_t* scratch_bytes) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!packed_bytes || !scratch_bytes) return fail(FF_ERR_ARG, "null output pointer");
    Plan P = make_plan(*cfg);
    *packed_bytes = P.packed_bytes;
    *scratch_bytes = P.scratch_bytes;
    return FF_OK;
}

int ff_model_create(const ff_config* cfg, void* packed_dev, size_t packed_bytes, void* scratch_dev, size_t scratch_bytes,
                    void* stream, ff_model** out) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!packed_dev || !scratch_dev || !out) return fail(FF_ERR_ARG, "null argument");
    if (((uintptr_t)packed_dev | (uintptr_t)scratch_dev) & 255) return fail(FF_ERR_NOMEM, "device buffers must be 256-byte aligned");
    Plan P = make_plan(*cfg);
    if (packed_bytes < P.packed_bytes) return fail(FF_ERR_NOMEM, "packed buffer too small: %zu < %zu", packed_bytes, P.packed_bytes);
    if (scratch_bytes < P.scratch_bytes) return fail(FF_ERR_NOMEM, "scratch buffer too small: %zu < %zu", scratch_bytes, P.scratch_bytes);
    hipStream_t st = (hipStream_t)stream;
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIPCHK(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return fail(FF_ERR_UNSUPPORTED, "device is %s, kernels are built for gfx950", prop.gcnArchName);

    ff_model* m = new (std::nothrow) ff_model();
    if (!m) return fail(FF_ERR_NOMEM, "host allocation failed");
    m->cfg = *cfg;
    m->plan = P;
    m->packed = (uint8_t*)packed_dev;
    m->scratch = (uint8_t*)scratch_dev;
    m->layer_loaded.assign(cfg->n_layers, 0);
    m->head_loaded = false;
    m->n_cta = prop.multiProcessorCount;
    m->lds_bytes = kLdsFusedBytes;
    if ((size_t)prop.sharedMemPerBlock < m->lds_bytes + 256) { delete m; return fail(FF_ERR_UNSUPPORTED, "device LDS per workgroup too small"); }
    if (fused_pass_rows(*cfg) == kMaxBatchWide && (!wide_fits(*cfg, m->n_cta) || m->n_cta > kGridCtas)) {
        delete m;
        return fail(FF_ERR_UNSUPPORTED, "max_batch %d needs the wide pass, whose row tiles do not fit a grid of %d workgroups", cfg->max_batch, prop.multiProcessorCount);
    }

    DevModel& D = m->dev;
    D.L = cfg->n_layers; D.d = cfg->d_model; D.Hq = cfg->n_q_heads; D.Hkv = cfg->n_kv_heads; D.hd = cfg->head_dim;
    D.F = cfg->d_ffn; D.V = cfg->vocab; D.eps = cfg->rms_eps;
    {   // gate/up pairs interleaved over the grid's waves when every wave owns the same whole number of
        // pairs and a staged K chunk of the down projection is a whole number of "one pair per wave" rounds
        const int nw = m->n_cta * kFusedWaves;
        const int chunk_elems = cfg->wdtype == W_BF16 ? kChunkUnitsOf<W_BF16> * 8 : cfg->wdtype == W_INT8 ? kChunkUnitsOf<W_INT8> * 16 : kChunkUnitsOf<W_INT4> * 32;
        // FF_GLU_PIPE: "0" keeps the two projections apart (A/B measurements), "all" also fuses them for int8
        // weights, where it measured slower (2.70 against 2.43 ms per step at the 8B shape: a wave's gate/up share
        // is only 14 stages long there, too few to stage the four chunks of h behind it) and is off by default
        const char* pipe = getenv("FF_GLU_PIPE");
        const bool pipe_off = pipe && pipe[0] == '0', pipe_all = pipe && pipe[0] == 'a';
        const bool ok = cfg->d_ffn % nw == 0 && chunk_elems % nw == 0 && !pipe_off;
        D.gu = ok ? GuPerm{cfg->d_ffn / nw, nw} : GuPerm{0, 0};
        // glu_run (single-sequence passes) needs the staged h beside the staged projection input, the
        // per-lane partial sums of a wave's down-projection rows at the end of the aux region, at most
        // kGluMaxChunks chunks and at least a ring's worth of gate/up stages per wave
        const int qd = cfg->n_q_heads * cfg->head_dim;
        const int in_off = (std::max(cfg->d_model, qd) + chunk_elems - 1) / chunk_elems * chunk_elems * 4;
        const int f_pad = (cfg->d_ffn + chunk_elems - 1) / chunk_elems * chunk_elems;
        const int pd = (cfg->d_model / 2 + nw - 1) / nw;                       // most down-projection row pairs a wave owns
        const int cpr_g = (cfg->d_model + chunk_elems - 1) / chunk_elems;      // stages per gate/up pair
        const bool fits = (size_t)in_off + (size_t)f_pad * 4 + (size_t)kFusedWaves * pd * 512 <= (size_t)kLdsActBytes + kLdsAuxBytes &&
                          f_pad / chunk_elems <= kGluMaxChunks && (cfg->d_ffn / nw) * cpr_g >= 4;
        m->glu_off = ok && fits && (cfg->wdtype != W_INT8 || pipe_all) ? in_off : -1;
    }
    D.layers = (const PLayer*)(m->packed + P.layers_tab);
    D.embed = (const bf16_t*)(m->packed + P.embed);
    D.gf = (const bf16_t*)(m->packed + P.gf);
    D.lm = to_pmat(P.lm, m->packed);
    uint8_t* s = m->scratch;
    D.x = (float*)(s + P.x); D.xn = (float*)(s + P.xn); D.q = (float*)(s + P.q); D.kvcur = (float*)(s + P.kvcur);
    D.attn_o = (float*)(s + P.attn_o); D.h = (float*)(s + P.h); D.y = (float*)(s + P.y);
    D.part_m = (float*)(s + P.part_m); D.part_l = (float*)(s + P.part_l); D.part_o = (float*)(s + P.part_o);
    D.status = (int*)(s + P.status);
    D.cx = (u32*)(s + P.cx); D.cx2 = (u32*)(s + P.cx2); D.cdelta = (u32*)(s + P.cdelta); D.tq = (u32x2*)(s + P.tq);
    D.tkvcur = (u32x2*)(s + P.tkvcur); D.cattn_o = (u32*)(s + P.cattn_o); D.ch = (u32*)(s + P.ch);
    D.wxres = (float*)(s + P.wxres); D.wimg_x = s + P.wimg_x; D.wimg_a = s + P.wimg_a; D.wimg_h = s + P.wimg_h;
    D.wsspart = (float*)(s + P.wsspart); D.wflag = (u32*)(s + P.wflag); D.wxch = (float*)(s + P.wxch); D.wpflag = (u32*)(s + P.wpflag);
    D.stepctr = (u32*)(s + P.stepctr);
    D.tpart_m = (u32x2*)(s + P.tpart_m); D.tpart_l = (u32x2*)(s + P.tpart_l); D.tpart_o = (u32x2*)(s + P.tpart_o);
    D.dbg = nullptr;
    for (int l = 0; l < cfg->n_layers; l++) {
        const LayerPlan& L = P.layers[l];
        PLayer pl;
        pl.g1 = (const bf16_t*)(m->packed + L.g1);
        pl.g2 = (const bf16_t*)(m->packed + L.g2);
        pl.qkv = to_pmat(L.qkv, m->packed); pl.o = to_pmat(L.o, m->packed);
        pl.gu = to_pmat(L.gu, m->packed); pl.down = to_pmat(L.down, m->packed);
        m->host_layers.push_back(pl);
    }
    hipError_t e = hipMemcpyAsync(m->packed + P.layers_tab, m->host_layers.data(), sizeof(PLayer) * cfg->n_layers, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) {
        k_fill_u32<<<256, 256, 0, st>>>((u32*)m->scratch, P.scratch_bytes / 4, 0u);
        // a model for single sequences never sees its batch grow: its one row is initialised here
        // and ff_decode_step launches no k_scrub_rows
        if (cfg->max_batch == 1) k_scrub_rows<<<64, kThreads, 0, st>>>(m->dev, 1);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);   // host_layers is pageable: finish the copy before returning
    if (e != hipSuccess) { delete m; return fail(FF_ERR_HIP, "model create: %s", hipGetErrorString(e)); }
    *out = m;
    return FF_OK;
}

int ff_model_load_layer(ff_model* m, int32_t layer, const ff_layer_weights* w, void* stream) {
    if (!m || !w) return fail(FF_ERR_ARG, "null argument");
    if (layer < 0 || layer >= m->cfg.n_layers) return fail(FF_ERR_ARG, "layer %d out of range", layer);
    if (!w->attn_norm || !w->ffn_norm) return fail(FF_ERR_ARG, "norm gain pointer is null");
    hipStream_t st = (hipStream_t)stream;
    const ff_config& c = m->cfg;
    const LayerPlan& L = m->plan.layers[layer];
    HIPCHK(hipMemcpyAsync(m->packed + L.g1, w->attn_norm, (size_t)c.d_model * 2, hipMemcpyDeviceToDevice, st));
    HIPCHK(hipMemcpyAsync(m->packed + L.g2, w->ffn_norm, (size_t)c.d_model * 2, hipMemcpyDeviceToDevice, st));
    int qr = c.n_q_heads * c.head_dim, kr = c.n_kv_heads * c.head_dim, rc;
    if ((rc = repack(L.qkv, m->packed, 0, qr, w->wq, nullptr, REPACK_ROPE, c.head_dim, m->dev.gu, st))) return rc;
    if ((rc = repack(L.qkv, m->packed, qr, kr, w->wk, nullptr, REPACK_ROPE, c.head_dim, m->dev.gu, st))) return rc;
    if ((rc = repack(L.qkv, m->packed, qr + kr, kr, w->wv, nullptr, REPACK_COPY, c.head_dim, m->dev.gu, st))) return rc;
    if ((rc = repack(L.o, m->packed, 0, c.d_model, w->wo, nullptr, REPACK_COPY, c.head_dim, m->dev.gu, st))) return rc;
    if ((rc = repack(L.gu, m->packed, 0, 2 * c.d_ffn, w->w_gate, &w->w_up, REPACK_INTERLEAVE, c.head_dim, m->dev.gu, st))) return rc;
    if ((rc = repack(L.down, m->packed, 0, c.d_model, w->w_down, nullptr, REPACK_COPY, c.head_dim, m->dev.gu, st))) return rc;
    m->layer_loaded[layer] = 1;
    return FF_OK;
}

int ff_model_load_head(ff_model* m, const ff_head_weights* w, void* stream) {
    if (!m || !w) return fail(FF_ERR_ARG, "null argument");
    if (!w->embed || !w->final_norm) return fail(FF_ERR_ARG, "embedding / final norm pointer is null");
    hipStream_t st = (hipStream_t)stream;
    const ff_config& c = m->cfg;
    HIPCHK(hipMemcpyAsync(m->packed + m->plan.embed, w->embed, (size_t)c.vocab * c.d_model * 2, hipMemcpyDeviceToDevice, st));
    HIPCHK(hipMemcpyAsync(m->packed + m->plan.gf, w->final_norm, (size_t)c.d_model * 2, hipMemcpyDeviceToDevice, st));
    int rc = repack(m->plan.lm, m->packed, 0, c.vocab, w->lm_head, nullptr, REPACK_COPY, c.head_dim, m->dev.gu, st);
    if (rc) return rc;
    m->head_loaded = true;
    return FF_OK;
}

int ff_model_load(const ff_config* cfg, const ff_layer_weights* layers, const ff_head_weights* head, void* packed_dev,
                  size_t packed_bytes, void* scratch_dev, size_t scratch_bytes, void* stream, ff_model** out) {
    if (!layers || !head) return fail(FF_ERR_ARG, "null argument");
    ff_model* m = nullptr;
    int rc = ff_model_create(cfg, packed_dev, packed_bytes, scratch_dev, scratch_bytes, stream, &m);
    if (rc) return rc;
    for (int l = 0; l < cfg->n_layers && !rc; l++) rc = ff_model_load_layer(m, l, &layers[l], stream);
    if (!rc) rc = ff_model_load_head(m, head, stream);
    if (rc) { delete m; return rc; }
    *out = m;
    return FF_OK;
}

}  // extern "C"

namespace {
// ---- the seeded recipe of the package's input generators, host part: tensor keys ----
uint32_t crc32_ieee(const char* s) {   // the common reflected CRC-32 (polynomial 0xEDB88320)
    uint32_t c = 0xFFFFFFFFu;
    for (; *s; ++s) {
        c ^= (uint8_t)*s;
        for (int b = 0; b < 8; b++) c = (c >> 1) ^ (0xEDB88320u & (0u - (c & 1u)));
    }
    return ~c;
}
uint32_t tensor_key(uint64_t seed, const char* fmt, ...) {
    char name[96];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(name, sizeof name, fmt, ap);
    va_end(ap);
    return (uint32_t)seed * 0x9E3779B1u + crc32_ieee(name);
}
constexpr double kIh4Std = 37837.22;   // std of the sum of four uniform 16-bit integers
SynthMat synth_mat(uint64_t seed, int layer, const char* which, int k, int wd) {
    SynthMat s;
    if (layer >= 0) {
        s.key_w = tensor_key(seed, "l%d.%s", layer, which);
        s.key_s = tensor_key(seed, "l%d.%s.s", layer, which);
        s.key_z = tensor_key(seed, "l%d.%s.z", layer, which);
    } else {
        s.key_w = tensor_key(seed, "%s", which);
        s.key_s = tensor_key(seed, "%s.s", which);
        s.key_z = tensor_key(seed, "%s.z", which);
    }
    s.k = k;
    s.c_scale = wd == W_INT8 ? (float)(0.02 / 73.6) : (float)(0.02 / 6.5);
    return s;
}
int synth_part(const MatPlan& dst, uint8_t* packed, int dst_row, int n_rows, const SynthMat& a, const SynthMat& b, int mode, int hd,
               const GuPerm& perm, hipStream_t st) {
    const size_t rb = dst.wd == W_BF16 ? (size_t)dst.k * 2 : dst.wd == W_INT8 ? (size_t)dst.k : (size_t)dst.k / 2;
    const size_t sb = dst.wd == W_INT8 ? 2 : (size_t)(dst.k / 128) * 2;
    k_synth_rows<<<std::min(n_rows, 8192), kThreads, 0, st>>>(packed + dst.w + (size_t)dst_row * rb, (f16_t*)(packed + dst.s + (size_t)dst_row * sb),
                                                             (f16_t*)(packed + dst.z + (size_t)dst_row * sb), n_rows, dst.wd, a, b, mode, hd,
                                                             (float)(0.02 / kIh4Std), perm);
    HIPCHK(hipGetLastError());
    return FF_OK;
}
}  // namespace

extern "C" {

int ff_model_load_synthetic(const ff_config* cfg, uint64_t seed, void* packed_dev, size_t packed_bytes, void* scratch_dev, size_t scratch_bytes,
                            void* stream, ff_model** out) {
    ff_model* m = nullptr;
    int rc = ff_model_create(cfg, packed_dev, packed_bytes, scratch_dev, scratch_bytes, stream, &m);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const ff_config& c = m->cfg;
    const int qr = c.n_q_heads * c.head_dim, kr = c.n_kv_heads * c.head_dim, wd = c.wdtype;
    const float gscale = (float)(0.02 / kIh4Std);
    for (int l = 0; l < c.n_layers && !rc; l++) {
        const LayerPlan& L = m->plan.layers[l];
        k_synth_normal<<<16, 256, 0, st>>>((bf16_t*)(m->packed + L.g1), (size_t)c.d_model, tensor_key(seed, "l%d.attn_norm", l), gscale, 1.0f);
        k_synth_normal<<<16, 256, 0, st>>>((bf16_t*)(m->packed + L.g2), (size_t)c.d_model, tensor_key(seed, "l%d.ffn_norm", l), gscale, 1.0f);
        const SynthMat wq = synth_mat(seed, l, "wq", c.d_model, wd), wk = synth_mat(seed, l, "wk", c.d_model, wd), wv = synth_mat(seed, l, "wv", c.d_model, wd),
                       wo = synth_mat(seed, l, "wo", qr, wd), wg = synth_mat(seed, l, "w_gate", c.d_model, wd), wu = synth_mat(seed, l, "w_up", c.d_model, wd),
                       wdn = synth_mat(seed, l, "w_down", c.d_ffn, wd);
        if (!rc) rc = synth_part(L.qkv, m->packed, 0, qr, wq, wq, REPACK_ROPE, c.head_dim, m->dev.gu, st);
        if (!rc) rc = synth_part(L.qkv, m->packed, qr, kr, wk, wk, REPACK_ROPE, c.head_dim, m->dev.gu, st);
        if (!rc) rc = synth_part(L.qkv, m->packed, qr + kr, kr, wv, wv, REPACK_COPY, c.head_dim, m->dev.gu, st);
        if (!rc) rc = synth_part(L.o, m->packed, 0, c.d_model, wo, wo, REPACK_COPY, c.head_dim, m->dev.gu, st);
        if (!rc) rc = synth_part(L.gu, m->packed, 0, 2 * c.d_ffn, wg, wu, REPACK_INTERLEAVE, c.head_dim, m->dev.gu, st);
        if (!rc) rc = synth_part(L.down, m->packed, 0, c.d_model, wdn, wdn, REPACK_COPY, c.head_dim, m->dev.gu, st);
        m->layer_loaded[l] = 1;
    }
    if (!rc) {
        k_synth_normal<<<2048, 256, 0, st>>>((bf16_t*)(m->packed + m->plan.embed), (size_t)c.vocab * c.d_model, tensor_key(seed, "embed"), gscale, 0.f);
        k_synth_normal<<<16, 256, 0, st>>>((bf16_t*)(m->packed + m->plan.gf), (size_t)c.d_model, tensor_key(seed, "final_norm"), gscale, 1.0f);
        const SynthMat lm = synth_mat(seed, -1, "lm_head", c.d_model, m->plan.lm.wd);
        rc = synth_part(m->plan.lm, m->packed, 0, c.vocab, lm, lm, REPACK_COPY, c.head_dim, m->dev.gu, st);
        m->head_loaded = true;
    }
    if (!rc && hipGetLastError() != hipSuccess) rc = fail(FF_ERR_HIP, "synthetic fill launch failed");
    if (rc) { delete m; return rc; }
    *out = m;
    return FF_OK;
}

int ff_model_free(ff_model* m) {
    delete m;
    return FF_OK;
}

int ff_kv_bytes(const ff_model* m, int32_t batch, int32_t max_ctx, size_t* bytes) {
    if (!m || !bytes) return fail(FF_ERR_ARG, "null argument");
    if (batch < 1 || batch > m->cfg.max_batch) return fail(FF_ERR_ARG, "batch %d outside [1,%d]", batch, m->cfg.max_batch);
    if (max_ctx < 1) return fail(FF_ERR_ARG, "max_ctx must be positive");
    if (max_ctx > (1 << 24)) return fail(FF_ERR_UNSUPPORTED, "max_ctx above 2^24 rows (the split arithmetic of the attention phase is 32-bit)");
    const ff_config& c = m->cfg;
    size_t cache = align256((size_t)c.n_layers * batch * c.n_kv_heads * 2 * (size_t)max_ctx * c.head_dim * 2);
    size_t rope = align256((size_t)max_ctx * (c.head_dim / 2) * sizeof(float2));
    *bytes = cache + rope;
    return FF_OK;
}

int ff_kv_alloc(ff_model* m, int32_t batch, int32_t max_ctx, void* kv_dev, size_t bytes, void* stream, ff_kv** out) {
    size_t need = 0;
    int rc = ff_kv_bytes(m, batch, max_ctx, &need);
    if (rc) return rc;
    if (!kv_dev || !out) return fail(FF_ERR_ARG, "null argument");
    if ((uintptr_t)kv_dev & 255) return fail(FF_ERR_NOMEM, "kv buffer must be 256-byte aligned");
    if (bytes < need) return fail(FF_ERR_NOMEM, "kv buffer too small: %zu < %zu", bytes, need);
    const ff_config& c = m->cfg;
    ff_kv* kv = new (std::nothrow) ff_kv();
    if (!kv) return fail(FF_ERR_NOMEM, "host allocation failed");
    kv->model = m; kv->batch = batch; kv->max_ctx = max_ctx;
    size_t cache = align256((size_t)c.n_layers * batch * c.n_kv_heads * 2 * (size_t)max_ctx * c.head_dim * 2);
    kv->dev.base = (bf16_t*)kv_dev;
    kv->dev.rope = (const float2*)((uint8_t*)kv_dev + cache);
    kv->dev.max_ctx = max_ctx; kv->dev.batch = batch; kv->dev.seq0 = 0; kv->dev.step_batch = batch;
    int n = max_ctx * (c.head_dim / 2);
    k_rope_table<<<(n + 255) / 256, 256, 0, (hipStream_t)stream>>>((float2*)kv->dev.rope, max_ctx, c.head_dim, (double)c.rope_theta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { delete kv; return fail(FF_ERR_HIP, "rope table: %s", hipGetErrorString(e)); }
    *out = kv;
    return FF_OK;
}

static int kv_copy(ff_kv* kv, int32_t layer, int32_t seq, int32_t pos0, int32_t n, void* k, void* v, void* stream, int dir) {
    if (!kv || !k || !v) return fail(FF_ERR_ARG, "null argument");
    const ff_config& c = kv->model->cfg;
    if (layer < 0 || layer >= c.n_layers || seq < 0 || seq >= kv->batch) return fail(FF_ERR_ARG, "layer/sequence index out of range");
    if (pos0 < 0 || n < 0 || (long)pos0 + n > kv->max_ctx) return fail(FF_ERR_RANGE, "rows [%d,%d) outside the cache (max_ctx %d)", pos0, pos0 + n, kv->max_ctx);
    if (n == 0) return FF_OK;
    size_t plane = (size_t)kv->max_ctx * c.head_dim;
    bf16_t* base = kv->dev.base + (((size_t)layer * kv->batch + seq) * c.n_kv_heads) * 2 * plane;
    size_t tot = (size_t)n * c.n_kv_heads * c.head_dim;
    int grid = (int)std::min<size_t>((tot + 255) / 256, 2048);
    k_kv_copy<<<grid, 256, 0, (hipStream_t)stream>>>(kv->dev, 0, c.n_kv_heads, c.head_dim, base, base + plane, 2 * plane, pos0, n,
                                                     (bf16_t*)k, (bf16_t*)v, dir);
    HIPCHK(hipGetLastError());
    return FF_OK;
}
int ff_kv_fill(ff_kv* kv, int32_t layer, int32_t seq, int32_t pos0, int32_t n, const void* k_dev, const void* v_dev, void* stream) {
    return kv_copy(kv, layer, seq, pos0, n, (void*)k_dev, (void*)v_dev, stream, 0);
}
int ff_kv_read(ff_kv* kv, int32_t layer, int32_t seq, int32_t pos0, int32_t n, void* k_dev, void* v_dev, void* stream) {
    return kv_copy(kv, layer, seq, pos0, n, k_dev, v_dev, stream, 1);
}
int ff_kv_fill_synthetic(ff_kv* kv, uint64_t seed, int32_t n_ctx, void* stream) {
    if (!kv) return fail(FF_ERR_ARG, "null argument");
    if (n_ctx < 0 || n_ctx > kv->max_ctx) return fail(FF_ERR_RANGE, "n_ctx %d outside [0, max_ctx %d]", n_ctx, kv->max_ctx);
    if (n_ctx == 0) return FF_OK;
    const ff_config& c = kv->model->cfg;
    const size_t plane = (size_t)kv->max_ctx * c.head_dim;
    const size_t tot = (size_t)n_ctx * c.n_kv_heads * c.head_dim;
    const int grid = (int)std::min<size_t>((tot + 255) / 256, 1024);
    for (int l = 0; l < c.n_layers; l++)
        for (int b = 0; b < kv->batch; b++) {
            bf16_t* base = kv->dev.base + (((size_t)l * kv->batch + b) * c.n_kv_heads) * 2 * plane;
            k_synth_kv<<<grid, 256, 0, (hipStream_t)stream>>>(base, plane, c.n_kv_heads, c.head_dim, n_ctx, tensor_key(seed, "kv.l%d.s%d.k", l, b),
                                                             tensor_key(seed, "kv.l%d.s%d.v", l, b), (float)(1.0 / kIh4Std));
        }
    HIPCHK(hipGetLastError());
    return FF_OK;
}

int ff_debug_stream_read(const void* buf_dev, size_t bytes, int32_t n_workgroups, void* stream) {
    if (!buf_dev || bytes < (size_t)1 << 20 || n_workgroups < 1 || n_workgroups > 65536) return fail(FF_ERR_ARG, "bad argument");
    if ((uintptr_t)buf_dev & 15) return fail(FF_ERR_ARG, "buffer must be 16-byte aligned");
    void* sink = nullptr;
    HIPCHK(hipGetSymbolAddress(&sink, HIP_SYMBOL(sink_word)));
    k_stream_read<<<n_workgroups, kThreads, 0, (hipStream_t)stream>>>((const u32x4*)buf_dev, bytes / 16, (u32*)sink);
    HIPCHK(hipGetLastError());
    return FF_OK;
}

int ff_kv_free(ff_kv* kv) {
    delete kv;
    return FF_OK;
}

namespace {
// One pass of the fused kernel over sequences [seq0, seq0 + batch) of a step of step_batch
// sequences, batch <= fused_pass_rows.  Nothing here depends on host-side state that changes from
// step to step (exchange tags, write counters and the rows to re-initialise all derive from
// counters kept on the device), so the launches of a step may be recorded into a HIP graph.
int fused_pass(ff_model* m, const DevModel& D, const int32_t* tokens_dev, const int32_t* positions_dev, ff_kv* kv, float* logits_dev, int32_t batch, int seq0,
               int step_batch, hipStream_t st) {
    const bool wide = pass_is_wide(m->cfg, batch);   // (batch <= fused_pass_rows: a wide pass only where the wide instance fits)
    // LM head inside the fused kernel when its weights have the layers' type: one phase, or with a
    // wide pass one phase per block of kDenseMaxTiles tiles per workgroup
    const int lm_block_rows = kDenseMaxTiles * 16 * m->n_cta;
    const int lm_in_kernel = D.lm.wd != m->cfg.wdtype ? 0 : wide ? (m->cfg.vocab + lm_block_rows - 1) / lm_block_rows : 1;
    DevKV kvd = kv->dev;
    kvd.seq0 = seq0;
    kvd.step_batch = step_batch;
    if (wide) {   // the step's embedding rows in the wide pass's exchange form
        k_wide_embed<<<m->n_cta, kThreads, 0, st>>>(D, tokens_dev, batch);
        HIPCHK(hipGetLastError());
    } else if (m->cfg.max_batch > 1) {   // rows a smaller batch left behind: see k_scrub_rows (decides on the device)
        k_scrub_rows<<<64, kThreads, 0, st>>>(D, batch);
        HIPCHK(hipGetLastError());
    }
    FusedLaunch a{D, kvd, tokens_dev, positions_dev, logits_dev, batch, lm_in_kernel, m->n_cta, m->lds_bytes, st, m->mute_wg, m->switches, m->glu_off,
                  wide ? 1 : 0};
    const char* what = "";
    const int G = m->cfg.n_q_heads / m->cfg.n_kv_heads;
    hipError_t e = hipErrorInvalidValue;
    what = "no fused kernel instance for this configuration";
#define FF_TRY_FAMILY(name, wd, hd, g) \
    if (m->cfg.wdtype == wd && m->cfg.head_dim == hd && G == g) e = launch_fused_##name##_hd##hd##_g##g(a, &what);
    FF_FUSED_FAMILIES(FF_TRY_FAMILY)
#undef FF_TRY_FAMILY
    if (e != hipSuccess) return fail(e == hipErrorLaunchOutOfResources ? FF_ERR_UNSUPPORTED : FF_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    if (!lm_in_kernel) {   // LM head of a different weight type than the layers: separate launches
        const ff_config& c = m->cfg;
        op_final_x<<<16, kThreads, 0, st>>>(D.x, D.cx, D.cdelta, batch * c.d_model);
        op_rmsnorm<<<batch, kThreads, 0, st>>>(D.x, D.gf, D.xn, c.d_model, c.rms_eps);
        for (int b0 = 0; b0 < batch; b0 += kMaxBatch) {
            int rc = gemv_op(m, D.lm, D.xn + (size_t)b0 * c.d_model, c.d_model, logits_dev + (size_t)b0 * c.vocab, std::min(kMaxBatch, batch - b0), EPI_STORE, st,
                             tokens_dev + b0);
            if (rc) return rc;
        }
        HIPCHK(hipGetLastError());
    }
    return FF_OK;
}
}  // namespace

// Batches above one pass run as consecutive passes on the stream (every pass streams the weights
// again; the exchange buffers are reused pass after pass).
int ff_decode_step(ff_model* m, const int32_t* tokens_dev, const int32_t* positions_dev, ff_kv* kv, float* logits_dev, int32_t batch,
                   void* stream) {
    int rc = check_step_args(m, tokens_dev, positions_dev, kv, logits_dev, batch);
    if (rc) return rc;
    const int rows = fused_pass_rows(m->cfg);
    for (int s0 = 0; s0 < batch; s0 += rows) {
        rc = fused_pass(m, m->dev, tokens_dev + s0, positions_dev + s0, kv, logits_dev + (size_t)s0 * m->cfg.vocab, std::min(rows, batch - s0),
                        s0, batch, (hipStream_t)stream);
        if (rc) return rc;
    }
    return FF_OK;
}

namespace {
int perop_pass(ff_model* m, const int32_t* tokens_dev, const int32_t* positions_dev, ff_kv* kv, float* logits_dev, int32_t batch, int seq0,
               int step_batch, hipStream_t st) {
    int rc = 0;
    DevKV kvd = kv->dev;
    kvd.seq0 = seq0;
    kvd.step_batch = step_batch;
    const DevModel& D = m->dev;
    const ff_config& c = m->cfg;
    static std::once_flag once;
    static int attr_rc = 0;
    std::call_once(once, [&] { attr_rc = set_lds(op_attn_partial, m->lds_bytes); });
    if (attr_rc) return fail(FF_ERR_HIP, "hipFuncSetAttribute failed for the attention kernel");
    const int qd = c.n_q_heads * c.head_dim, qkv_rows = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    const int share = std::max(1, m->n_cta / (batch * c.n_kv_heads));
    const int ew_grid = 64;
    op_embed<<<ew_grid, kThreads, 0, st>>>(D, kvd, tokens_dev, positions_dev, batch);
    for (int l = 0; l < c.n_layers; l++) {
        const PLayer& L = m->host_layers[l];
        op_rmsnorm<<<batch, kThreads, 0, st>>>(D.x, L.g1, D.xn, c.d_model, c.rms_eps);
        if ((rc = gemv_op(m, L.qkv, D.xn, c.d_model, D.y, batch, EPI_STORE, st))) return rc;
        op_rope_append<<<ew_grid, kThreads, 0, st>>>(D, kvd, tokens_dev, positions_dev, batch, l);
        op_attn_partial<<<m->n_cta, kThreads, m->lds_bytes, st>>>(D, kvd, tokens_dev, positions_dev, batch, l);
        op_attn_merge<<<batch * c.n_kv_heads, kThreads, 0, st>>>(D, kvd, tokens_dev, positions_dev, batch, share);
        if ((rc = gemv_op(m, L.o, D.attn_o, qd, D.x, batch, EPI_RESIDUAL, st))) return rc;
        op_rmsnorm<<<batch, kThreads, 0, st>>>(D.x, L.g2, D.xn, c.d_model, c.rms_eps);
        if ((rc = gemv_op(m, L.gu, D.xn, c.d_model, D.y, batch, EPI_STORE, st))) return rc;
        op_swiglu<<<ew_grid, kThreads, 0, st>>>(D, batch);
        if ((rc = gemv_op(m, L.down, D.h, c.d_ffn, D.x, batch, EPI_RESIDUAL, st))) return rc;
    }
    op_rmsnorm<<<batch, kThreads, 0, st>>>(D.x, D.gf, D.xn, c.d_model, c.rms_eps);
    if ((rc = gemv_op(m, D.lm, D.xn, c.d_model, logits_dev, batch, EPI_STORE, st, tokens_dev))) return rc;
    (void)qkv_rows;
    HIPCHK(hipGetLastError());
    return FF_OK;
}
}  // namespace

int ff_decode_step_perop(ff_model* m, const int32_t* tokens_dev, const int32_t* positions_dev, ff_kv* kv, float* logits_dev,
                         int32_t batch, void* stream) {
    int rc = check_step_args(m, tokens_dev, positions_dev, kv, logits_dev, batch);
    if (rc) return rc;
    for (int s0 = 0; s0 < batch; s0 += kMaxBatch) {
        rc = perop_pass(m, tokens_dev + s0, positions_dev + s0, kv, logits_dev + (size_t)s0 * m->cfg.vocab, std::min(kMaxBatch, batch - s0), s0,
                        batch, (hipStream_t)stream);
        if (rc) return rc;
    }
    return FF_OK;
}

}  // extern "C"

namespace {
// Device address of this GPU's copy of the static scratch array (looked up once per device).
int static_scratch_ptr(uint8_t** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static uint8_t* ptrs[kMaxDevices] = {};
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(FF_ERR_UNSUPPORTED, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
        HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255)) return fail(FF_ERR_HIP, "static scratch array has no usable device address");
        ptrs[dev] = (uint8_t*)p;
    }
    *out = ptrs[dev];
    return FF_OK;
}
}  // namespace

extern "C" {

int ff_decode_step_static(ff_model* m, const int32_t* tokens_dev, const int32_t* positions_dev, ff_kv* kv, float* logits_dev, int32_t batch,
                          void* stream) {
    int rc = check_step_args(m, tokens_dev, positions_dev, kv, logits_dev, batch);
    if (rc) return rc;
    const Plan& P = m->plan;
    if (P.scratch_bytes > kStaticScratchBytes)
        return fail(FF_ERR_NOMEM, "this configuration needs %zu bytes of exchange scratch, the static array holds %zu", P.scratch_bytes,
                    kStaticScratchBytes);
    uint8_t* s = nullptr;
    if ((rc = static_scratch_ptr(&s))) return rc;
    hipStream_t st = (hipStream_t)stream;
    // the model's exchange pointers moved onto the static array (same layout); the status word and
    // the optional timeline stay with the model, where ff_status looks for them
    DevModel D = m->dev;
    D.x = (float*)(s + P.x); D.xn = (float*)(s + P.xn); D.q = (float*)(s + P.q); D.kvcur = (float*)(s + P.kvcur);
    D.attn_o = (float*)(s + P.attn_o); D.h = (float*)(s + P.h); D.y = (float*)(s + P.y);
    D.part_m = (float*)(s + P.part_m); D.part_l = (float*)(s + P.part_l); D.part_o = (float*)(s + P.part_o);
    D.cx = (u32*)(s + P.cx); D.cx2 = (u32*)(s + P.cx2); D.cdelta = (u32*)(s + P.cdelta); D.tq = (u32x2*)(s + P.tq);
    D.tkvcur = (u32x2*)(s + P.tkvcur); D.cattn_o = (u32*)(s + P.cattn_o); D.ch = (u32*)(s + P.ch);
    D.wxres = (float*)(s + P.wxres); D.wimg_x = s + P.wimg_x; D.wimg_a = s + P.wimg_a; D.wimg_h = s + P.wimg_h;
    D.wsspart = (float*)(s + P.wsspart); D.wflag = (u32*)(s + P.wflag); D.wxch = (float*)(s + P.wxch); D.wpflag = (u32*)(s + P.wpflag);
    D.stepctr = (u32*)(s + P.stepctr);
    D.tpart_m = (u32x2*)(s + P.tpart_m); D.tpart_l = (u32x2*)(s + P.tpart_l); D.tpart_o = (u32x2*)(s + P.tpart_o);
    // The array keeps whatever the last call (of any model) left: everything this step's kernels
    // test before they write it is cleared first -- tags and step counter to zero (a fill kernel,
    // not a memset node, so the call may be recorded into a HIP graph), then the write-counter
    // bits of the compact rows (k_scrub_rows sees "0 rows clean").
    k_fill_u32<<<256, 256, 0, st>>>((u32*)s, P.scratch_bytes / 4, 0u);
    k_scrub_rows<<<64, kThreads, 0, st>>>(D, std::min(batch, fused_pass_rows(m->cfg)));
    HIPCHK(hipGetLastError());
    const int rows = fused_pass_rows(m->cfg);
    for (int s0 = 0; s0 < batch; s0 += rows) {
        rc = fused_pass(m, D, tokens_dev + s0, positions_dev + s0, kv, logits_dev + (size_t)s0 * m->cfg.vocab, std::min(rows, batch - s0), s0,
                        batch, st);
        if (rc) return rc;
    }
    return FF_OK;
}

int ff_status(ff_model* m, void* stream) {
    if (!m) return fail(FF_ERR_ARG, "null argument");
    hipStream_t st = (hipStream_t)stream;
    HIPCHK(hipStreamSynchronize(st));
    int s = 0;
    HIPCHK(hipMemcpy(&s, m->dev.status, sizeof(int), hipMemcpyDeviceToHost));
    if (s != 0) {
        HIPCHK(hipMemset(m->dev.status, 0, sizeof(int)));
        if (s == kStatusRange) return fail(FF_ERR_RANGE, "a decode step saw a position outside [0, max_ctx) or a token id that is neither in [0, vocab) nor FF_TOKEN_SKIP, and was skipped");
        if (s <= -50 || s == kStatusTimeout)
            return fail(FF_ERR_TIMEOUT, "a workgroup gave up waiting for another workgroup's output (site code %d): workgroups not co-resident?", s);
        return fail(FF_ERR_HIP, "unknown device status %d", s);
    }
    return FF_OK;
}

}  // extern "C"

namespace {
// Which packed matrix holds canonical matrix `which`, and how canonical rows map to packed rows.
struct MatSel { PMat W; int n_can, map, parity, row_off; };
int select_matrix(const ff_model* m, int32_t layer, int32_t which, MatSel* out) {
    const ff_config& c = m->cfg;
    if (which != FF_MAT_LMHEAD && (layer < 0 || layer >= c.n_layers)) return fail(FF_ERR_ARG, "layer %d out of range", layer);
    const int qr = c.n_q_heads * c.head_dim, kr = c.n_kv_heads * c.head_dim;
    const PLayer* L = which == FF_MAT_LMHEAD ? nullptr : &m->host_layers[layer];
    MatSel s{};
    switch (which) {
        case FF_MAT_WQ: s.W = L->qkv; s.n_can = qr; s.map = 1; break;
        case FF_MAT_WK: s.W = L->qkv; s.n_can = kr; s.map = 1; s.row_off = qr; break;
        case FF_MAT_WV: s.W = L->qkv; s.n_can = kr; s.row_off = qr + kr; break;
        case FF_MAT_WO: s.W = L->o; s.n_can = c.d_model; break;
        case FF_MAT_WGATE: s.W = L->gu; s.n_can = c.d_ffn; s.map = 2; s.parity = 0; break;
        case FF_MAT_WUP: s.W = L->gu; s.n_can = c.d_ffn; s.map = 2; s.parity = 1; break;
        case FF_MAT_WDOWN: s.W = L->down; s.n_can = c.d_model; break;
        case FF_MAT_LMHEAD: s.W = m->dev.lm; s.n_can = c.vocab; break;
        default: return fail(FF_ERR_ARG, "unknown matrix id %d", which);
    }
    *out = s;
    return FF_OK;
}
template <int WD, int B>
int launch_debug_quad(ff_model* m, const PMat& W, const float* in, float* out, int batch, hipStream_t st) {
    auto kern = k_debug_gemv_quad<WD, B>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] { attr_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)m->lds_bytes); });
    if (attr_err != hipSuccess) return fail(FF_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(attr_err));
    kern<<<m->n_cta, kThreads, m->lds_bytes, st>>>(W, in, W.k, out, batch);
    return FF_OK;
}
template <int WD>
int debug_quad_any(ff_model* m, const PMat& W, const float* in, float* out, int batch, hipStream_t st) {
    if (batch == 2) return launch_debug_quad<WD, 2>(m, W, in, out, batch, st);
    return launch_debug_quad<WD, 4>(m, W, in, out, batch, st);
}
}  // namespace

extern "C" {

int ff_debug_gemv(ff_model* m, int32_t layer, int32_t which, const float* in_dev, float* out_dev, int32_t batch, int32_t path, void* stream) {
    if (!m || !in_dev || !out_dev) return fail(FF_ERR_ARG, "null argument");
    if (path != 0 && path != 1) return fail(FF_ERR_ARG, "path must be 0 (vector ALU) or 1 (matrix cores)");
    const int max_rows = std::min(m->cfg.max_batch, kMaxBatch);
    if (batch < 1 || batch > max_rows || (path == 1 && batch < 2)) return fail(FF_ERR_ARG, "batch %d not served by this path (model max_batch %d)", batch, m->cfg.max_batch);
    MatSel s;
    int rc = select_matrix(m, layer, which, &s);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const PMat& W = s.W;
    const int epu = W.wd == W_BF16 ? 8 : W.wd == W_INT8 ? 16 : 32;
    if (path == 1 && (size_t)W.k * 4 * (size_t)(batch <= 2 ? 2 : 4) > (size_t)kLdsActBytes)
        return fail(FF_ERR_UNSUPPORTED, "matrix-core debug GEMV needs the input rows in one K segment (K = %d)", W.k);
    (void)epu;
    // raw output in packed row order: straight into out_dev when rows need no mapping and the matrix
    // is not shared (LM head, output and down projections), else through the per-op row buffer
    const bool direct = s.map == 0 && s.row_off == 0 && W.n == s.n_can;
    float* raw = direct ? out_dev : m->dev.y;
    if (path == 0) rc = gemv_op(m, W, in_dev, W.k, raw, batch, EPI_STORE, st);
    else if (W.wd == W_BF16) rc = debug_quad_any<W_BF16>(m, W, in_dev, raw, batch, st);
    else if (W.wd == W_INT8) rc = debug_quad_any<W_INT8>(m, W, in_dev, raw, batch, st);
    else rc = debug_quad_any<W_INT4>(m, W, in_dev, raw, batch, st);
    if (rc) return rc;
    if (!direct) k_unmap_rows<<<256, 256, 0, st>>>(raw, W.n, out_dev, s.n_can, s.map, s.parity, s.row_off, m->cfg.head_dim, batch, m->dev.gu);
    HIPCHK(hipGetLastError());
    return FF_OK;
}

int ff_debug_dequant(const ff_model* m, int32_t layer, int32_t which, float* out_dev, void* stream) {
    if (!m || !out_dev) return fail(FF_ERR_ARG, "null argument");
    MatSel s;
    int rc = select_matrix(m, layer, which, &s);
    if (rc) return rc;
    k_dequant<<<2048, 256, 0, (hipStream_t)stream>>>(s.W, out_dev, s.n_can, s.map, s.parity, s.row_off, m->cfg.head_dim, m->dev.gu);
    HIPCHK(hipGetLastError());
    return FF_OK;
}

int ff_debug_timeline(ff_model* m, void* buf_dev) {
    if (!m) return fail(FF_ERR_ARG, "null argument");
    m->dev.dbg = (u64*)buf_dev;
    return FF_OK;
}

}  // extern "C"

namespace {
template <bool OVERLAP>
int launch_stack(const StackArgs& a, int n_cta, hipStream_t st) {
    auto kern = stack_linear_kernel<OVERLAP>;
    static std::once_flag once;
    static hipError_t setup_err = hipSuccess;
    std::call_once(once, [&] {
        setup_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsFusedBytes);
        int occ = 0;
        if (setup_err == hipSuccess) setup_err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kern, kFusedThreads, kLdsFusedBytes);
        if (setup_err == hipSuccess && occ < 1) setup_err = hipErrorLaunchOutOfResources;
    });
    if (setup_err != hipSuccess) return fail(FF_ERR_HIP, "stacked-linear kernel set-up failed: %s", hipGetErrorString(setup_err));
    kern<<<n_cta, kFusedThreads, kLdsFusedBytes, st>>>(a, n_cta);
    return FF_OK;
}
}  // namespace

extern "C" {

int ff_debug_stack_linear(const void* w_dev, int32_t d, int32_t n_layers, const float* x_dev, float* y_dev, int32_t mode, void* scratch_dev,
                          size_t scratch_bytes, void* stream) {
    if (!w_dev || !x_dev || !y_dev || !scratch_dev) return fail(FF_ERR_ARG, "null argument");
    if (mode < 0 || mode > 2) return fail(FF_ERR_ARG, "mode must be 0 (one launch per layer), 1 (fused) or 2 (fused + overlap)");
    // every wave of the grid must own rows of every layer (d / 2 row pairs over 1024 waves) and the staged
    // vector must be a whole number of tile chunks
    if (d < 2048 || d % 2048 || (size_t)d * 4 > (size_t)kLdsActBytes || n_layers < 1 || n_layers > 4096)
        return fail(FF_ERR_UNSUPPORTED, "d must be a multiple of 2048 in [2048, 32768], n_layers in [1, 4096]");
    const size_t need = 2 * align256((size_t)d * 4) + 256;
    if (scratch_bytes < need || ((uintptr_t)scratch_dev & 255)) return fail(FF_ERR_NOMEM, "scratch needs %zu bytes, 256-byte aligned", need);
    hipStream_t st = (hipStream_t)stream;
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    int n_cta = 0;
    HIPCHK(hipDeviceGetAttribute(&n_cta, hipDeviceAttributeMultiprocessorCount, dev));
    uint8_t* s = (uint8_t*)scratch_dev;
    if (mode == 0) {
        // plain fp32 vectors ping-pong in the scratch; one streaming-GEMV launch per layer
        float* b0 = (float*)s;
        float* b1 = (float*)(s + align256((size_t)d * 4));
        HIPCHK(hipMemcpyAsync(b0, x_dev, (size_t)d * 4, hipMemcpyDeviceToDevice, st));
        ff_model shim;   // launch_gemv only needs the launch shape
        shim.n_cta = n_cta; shim.lds_bytes = kLdsFusedBytes;
        for (int l = 0; l < n_layers; l++) {
            PMat W;
            W.w = (const uint8_t*)w_dev + (size_t)l * d * d * 2; W.s = nullptr; W.z = nullptr; W.n = d; W.k = d; W.wd = W_BF16;
            int rc = launch_gemv<W_BF16, 1>(&shim, W, (l & 1) ? b1 : b0, d, (l & 1) ? b0 : b1, 1, EPI_STORE, st);
            if (rc) return rc;
        }
        HIPCHK(hipMemcpyAsync(y_dev, (n_layers & 1) ? b1 : b0, (size_t)d * 4, hipMemcpyDeviceToDevice, st));
        HIPCHK(hipGetLastError());
        return FF_OK;
    }
    StackArgs a;
    a.w = (const uint8_t*)w_dev; a.d = d; a.n_layers = n_layers;
    a.buf[0] = (cword_t*)s; a.buf[1] = (cword_t*)(s + align256((size_t)d * 4));
    a.status = (int*)(s + 2 * align256((size_t)d * 4));
    k_stack_pack<<<16, 256, 0, st>>>(a, x_dev);
    int rc = mode == 2 ? launch_stack<true>(a, n_cta, st) : launch_stack<false>(a, n_cta, st);
    if (rc) return rc;
    k_stack_unpack<<<16, 256, 0, st>>>(a, y_dev);
    HIPCHK(hipGetLastError());
    return FF_OK;
}

int ff_debug_set_overlap(ff_model* m, int32_t overlap) {
    if (!m) return fail(FF_ERR_ARG, "null argument");
    if (!overlap && (m->cfg.wdtype != W_BF16 || m->cfg.max_batch != 1))
        return fail(FF_ERR_UNSUPPORTED, "the no-overlap variant exists for bf16 models with max_batch 1 only");
    m->switches = overlap ? (m->switches & ~kSwNoOverlap) : (m->switches | kSwNoOverlap);
    return FF_OK;
}

int ff_debug_set_attention_balance(ff_model* m, int32_t by_length) {
    if (!m) return fail(FF_ERR_ARG, "null argument");
    m->switches = by_length ? (m->switches & ~kSwUniformShares) : (m->switches | kSwUniformShares);
    return FF_OK;
}

int ff_debug_mute_workgroup(ff_model* m, int32_t workgroup) {
    if (!m) return fail(FF_ERR_ARG, "null argument");
    if (workgroup < -1 || workgroup >= m->n_cta) return fail(FF_ERR_ARG, "workgroup %d outside [-1, %d)", workgroup, m->n_cta);
    m->mute_wg = workgroup;
    return FF_OK;
}

int ff_fused_schedule(const ff_model* m, int32_t* barriers_per_step, int32_t* n_workgroups, int32_t* threads_per_workgroup) {
    if (!m) return fail(FF_ERR_ARG, "null argument");
    if (barriers_per_step) *barriers_per_step = 0;   // phases are ordered by tagged dataflow, not by grid barriers
    if (n_workgroups) *n_workgroups = m->n_cta;
    if (threads_per_workgroup) *threads_per_workgroup = kFusedThreads;
    return FF_OK;
}

}  // extern "C"
