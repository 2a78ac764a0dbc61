// C-ABI host layer: argument validation, launch planning, dispatch. No device
// memory is allocated or freed here and nothing synchronises; see include/lasp.h.
#include "../../include/lasp.h"
#include "../../include/lasp_profile.h"

#include <cmath>
#include <cstdint>
#include <mutex>
#include <utility>
#include <vector>

#include "lasp_internal.h"

namespace {

// Segments per head when the caller leaves the choice to the library: enough
// workgroups (B*H*segments) to fill a 256-CU device at the residency of the
// walking kernel of each pass (forward: two 4-wave workgroups per CU; backward
// on bfloat16: one 8-wave workgroup per CU), never more than one per tile.
constexpr int kTargetWorkgroupsFwd = 512;
constexpr int kTargetWorkgroupsBwd = 256;
enum Pass { kForward = 0, kBackward = 1 };

bool valid_dims(const lasp_shape *s) {
    if (!s) return false;
    if (s->B <= 0 || s->H <= 0 || s->N <= 0) return false;
    if (s->D != 64 && s->D != 128) return false;
    if (s->chunk != 64 && s->chunk != 128 && s->chunk != 256) return false;
    if ((int64_t)s->B * s->H > 65535) return false;  // grid.y limit
    if (s->kv_heads < 0 || (s->kv_heads > 0 && (s->kv_heads > s->H || s->H % s->kv_heads != 0))) return false;
    if (s->Dv != 0 && s->Dv != 64 && s->Dv != 128) return false;
    return true;
}

int make_plan(const lasp_shape *s, Pass pass, lasp::Plan *p, bool token = false, bool norm = false) {
    if (!s) return LASP_ERR_NULL;
    if (s->dtype != LASP_F32 && s->dtype != LASP_BF16) return LASP_ERR_DTYPE;
    if (!valid_dims(s)) return LASP_ERR_SHAPE;
    p->B = s->B;
    p->H = s->H;
    p->N = s->N;
    p->dk = s->D;
    p->dv = s->Dv != 0 ? s->Dv : s->D;
    p->D = p->dk > p->dv ? p->dk : p->dv;   // the kernels' dimension; the narrower of the two is zero-padded on chip
    p->dtype = s->dtype;
    p->kvdiv = s->kv_heads > 0 ? s->H / s->kv_heads : 1;
    p->tile = lasp::tile_tokens(s->dtype, s->chunk, p->D);
    p->ntiles = (s->N + p->tile - 1) / p->tile;
    // A short last tile is handled by the per-token-decay kernels only: with one lambda per head the
    // library synthesises log g = log(lambda) and runs those (with or without the fused Norm).
    const bool ragged = s->N % p->tile != 0;
    p->synth = ragged && !token;
    if (p->synth) token = true;
    int want = s->segments;
    if (want < 0 || want > p->ntiles) return LASP_ERR_SHAPE;
    if (want == 0) {
        int64_t chains = (int64_t)s->B * s->H;
        const int target = (pass == kBackward && s->dtype == LASP_BF16) ? kTargetWorkgroupsBwd : kTargetWorkgroupsFwd;
        want = (int)((target + chains - 1) / chains);
        if (want > p->ntiles) want = p->ntiles;
        if (want < 1) want = 1;
    }
    p->token = token;
    p->norm = norm;
    p->cache_stride = lasp::cache_stride_for(p->dtype, p->tile, p->ntiles, token, p->dk != p->dv);
    p->tiles_per_seg = (p->ntiles + want - 1) / want;
    if (p->cache_stride == 2) p->tiles_per_seg += p->tiles_per_seg & 1;   // segments start on cached tiles
    p->nseg = (p->ntiles + p->tiles_per_seg - 1) / p->tiles_per_seg;  // every segment non-empty
    return LASP_OK;
}

size_t elem_bytes(int dtype) { return dtype == LASP_F32 ? 4 : 2; }

size_t cache_bytes(const lasp_shape *shape, bool token) {
    lasp::Plan p;
    if (make_plan(shape, kForward, &p, token) != LASP_OK) return 0;
    // (a synthesised plan has token == true and the same cache stride rule)
    return (size_t)p.B * p.H * (p.ntiles / p.cache_stride) * p.dk * p.dv * elem_bytes(p.dtype);   // [d_k][d_v] per slot
}

// Scratch layout: [segment states][per-token decay only: segment log-decays][.. : per-token r_t]
// [synthesised log g only: log g per token][grouped K/V heads only: dK, dV per query head].
struct ScratchLayout {
    size_t states, seglog, rtok, logg, dk_part, dv_part, total;  // byte offsets of the regions (states = 0), total size
};
size_t round256(size_t x) { return (x + 255) / 256 * 256; }
bool scratch_layout(const lasp_shape *shape, bool token, ScratchLayout *l) {
    lasp::Plan f, b;
    if (make_plan(shape, kForward, &f, token) != LASP_OK || make_plan(shape, kBackward, &b, token) != LASP_OK) return false;
    const size_t nseg = f.nseg > b.nseg ? f.nseg : b.nseg;  // one buffer serves both passes
    const size_t chains = (size_t)f.B * f.H;
    l->states = 0;
    l->seglog = round256(chains * nseg * f.dk * f.dv * sizeof(float));   // segment states, [d_k][d_v] floats each
    l->rtok = l->logg = l->seglog;
    size_t end = l->seglog;
    if (f.token) {   // requested, or synthesised for a short last tile
        const size_t per_token = round256(chains * (size_t)f.N * sizeof(float));
        l->rtok = l->seglog + round256(chains * nseg * sizeof(float));
        l->logg = l->rtok + per_token;
        end = l->logg + (f.synth ? per_token : 0);
    }
    l->dk_part = l->dv_part = end;
    if (f.kvdiv > 1) {
        l->dv_part = l->dk_part + round256(chains * (size_t)f.N * f.dk * elem_bytes(f.dtype));
        end = l->dv_part + round256(chains * (size_t)f.N * f.dv * elem_bytes(f.dtype));
    }
    l->total = end;
    return true;
}

// Event pool of the diagnostic profiler (lasp_profile_begin / lasp_profile_end).
struct Profiler {
    bool on = false;
    int cap = 0;
    int used[2] = {0, 0};                       // recorded forward / backward calls
    std::vector<lasp::KernelEvents> slots[2];
} g_prof;

const lasp::KernelEvents *next_slot(int kind) {
    if (!g_prof.on || g_prof.used[kind] >= g_prof.cap) return nullptr;
    return &g_prof.slots[kind][g_prof.used[kind]++];
}

struct Span {
    const void *p;
    size_t n;
};
bool overlap(Span a, Span b) {
    const char *x = (const char *)a.p, *y = (const char *)b.p;
    return x && y && x < y + b.n && y < x + a.n;
}

// Outputs must not overlap inputs or each other, and the kernels move data in 16-byte pieces.
// NULL (an absent optional buffer) passes both checks.
int check_buffers(const std::vector<Span> &ins, const std::vector<Span> &outs) {
    for (const Span &x : ins)
        if ((uintptr_t)x.p % 16 != 0) return LASP_ERR_ALIGN;
    for (const Span &x : outs)
        if ((uintptr_t)x.p % 16 != 0) return LASP_ERR_ALIGN;
    for (const Span &o : outs) {
        for (const Span &i : ins)
            if (overlap(o, i)) return LASP_ERR_ALIAS;
        for (const Span &o2 : outs)
            if (&o != &o2 && overlap(o, o2)) return LASP_ERR_ALIAS;
    }
    return LASP_OK;
}

// One forward call of any flavour: `token` selects the decay model (decay = lambda [H] or log g
// [B][H][N]), `norm` the fused output normalisation (eps, rstd).
struct FwdCall {
    const lasp_shape *shape;
    const void *q, *k, *v;
    const float *kv_in, *decay;
    bool token, norm;
    float eps;
    void *out;
    float *rstd, *kv_out;
    void *cache, *scratch;
    size_t scratch_bytes;
    void *stream;
};

int run_fwd_call(const FwdCall &c) {
    lasp::Plan p;
    int rc = make_plan(c.shape, kForward, &p, c.token, c.norm);
    if (rc != LASP_OK) return rc;
    if (!c.q || !c.k || !c.v || !c.decay || !c.out || !c.kv_out || (c.norm && !c.rstd)) return LASP_ERR_NULL;
    if (c.norm && (!std::isfinite(c.eps) || c.eps < 0.0f)) return LASP_ERR_SHAPE;
    ScratchLayout l;
    scratch_layout(c.shape, c.token, &l);
    if (!c.scratch || c.scratch_bytes < l.total) return LASP_ERR_WORKSPACE;

    const size_t esz = elem_bytes(p.dtype);
    const size_t qb = (size_t)p.B * p.H * p.N * p.dk * esz, ob = (size_t)p.B * p.H * p.N * p.dv * esz;   // q / out
    const size_t sb = (size_t)p.B * p.H * p.dk * p.dv * sizeof(float);
    const size_t gb = (size_t)p.B * p.H * p.N * sizeof(float);
    rc = check_buffers({{c.q, qb}, {c.k, qb / p.kvdiv}, {c.v, ob / p.kvdiv}, {c.kv_in, sb},
                        {c.decay, c.token ? gb : p.H * sizeof(float)}},
                       {{c.out, ob}, {c.rstd, gb}, {c.kv_out, sb}, {c.cache, cache_bytes(c.shape, c.token)},
                        {c.scratch, l.total}});
    if (rc != LASP_OK) return rc;

    hipStream_t stream = (hipStream_t)c.stream;
    char *scr = (char *)c.scratch;
    lasp::FwdArgs a{c.q, c.k, c.v, c.kv_in, c.decay, c.out, c.kv_out, c.cache, (float *)scr,
                    p.token ? (float *)(scr + l.seglog) : nullptr, c.rstd, c.eps, false};
    if (p.synth) {
        float *lg = (float *)(scr + l.logg);
        if (lasp::launch_fill_logg(p, c.decay, lg, stream) != hipSuccess) return LASP_ERR_HIP;
        a.decay = lg;
    }
    return lasp::launch_fwd(p, a, stream, next_slot(0)) == hipSuccess ? LASP_OK : LASP_ERR_HIP;
}

// One backward call of any flavour. `yn`, `rstd`: norm only; `kv_out`, `dlog_g`: per-token decay only.
struct BwdCall {
    const lasp_shape *shape;
    const void *q, *k, *v, *dout;
    const float *kv_in;     // used only when cache is NULL (the states are then rebuilt from it); NULL = zeros
    const float *dkv_out, *decay;
    bool token, norm;
    const void *yn;
    const float *rstd, *kv_out;
    const void *cache;
    void *dq, *dk, *dv;
    float *dlog_g, *dkv_in;
    void *scratch;
    size_t scratch_bytes;
    void *stream;
};

// Without a state cache the backward pass rebuilds the states first (Sec. 3.4: recomputation instead of
// caching): the forward pass reduced to its states writes them into the tail of the scratch buffer.
size_t recompute_scratch(const lasp_shape *shape, bool token) {
    ScratchLayout l;
    if (!scratch_layout(shape, token, &l)) return 0;
    return round256(l.total) + cache_bytes(shape, token);
}

int run_bwd_call(const BwdCall &c) {
    lasp::Plan p;
    int rc = make_plan(c.shape, kBackward, &p, c.token, c.norm);
    if (rc != LASP_OK) return rc;
    if (!c.q || !c.k || !c.v || !c.dout || !c.decay || !c.dq || !c.dk || !c.dv || !c.dkv_in)
        return LASP_ERR_NULL;
    if (c.norm && (!c.yn || !c.rstd)) return LASP_ERR_NULL;
    if (c.token && (!c.dlog_g || (c.dkv_out && !c.kv_out))) return LASP_ERR_NULL;
    ScratchLayout l;
    scratch_layout(c.shape, c.token, &l);
    const bool rebuild = c.cache == nullptr;
    const size_t cb = cache_bytes(c.shape, c.token);
    const size_t need = rebuild ? round256(l.total) + cb : l.total;
    if (!c.scratch || c.scratch_bytes < need) return LASP_ERR_WORKSPACE;
    char *scr = (char *)c.scratch;
    const void *cache = rebuild ? scr + round256(l.total) : c.cache;

    const size_t esz = elem_bytes(p.dtype);
    const size_t qb = (size_t)p.B * p.H * p.N * p.dk * esz, ob = (size_t)p.B * p.H * p.N * p.dv * esz;   // q / out
    const size_t sb = (size_t)p.B * p.H * p.dk * p.dv * sizeof(float);
    const size_t gb = (size_t)p.B * p.H * p.N * sizeof(float);
    rc = check_buffers({{c.q, qb}, {c.k, qb / p.kvdiv}, {c.v, ob / p.kvdiv}, {c.dout, ob}, {c.dkv_out, sb}, {c.kv_out, sb},
                        {rebuild ? c.kv_in : nullptr, sb}, {c.yn, ob}, {c.rstd, gb}, {c.decay, c.token ? gb : p.H * sizeof(float)},
                        {c.cache, cb}},
                       {{c.dq, qb}, {c.dk, qb / p.kvdiv}, {c.dv, ob / p.kvdiv}, {c.dlog_g, gb}, {c.dkv_in, sb},
                        {c.scratch, need}});
    if (rc != LASP_OK) return rc;

    hipStream_t stream = (hipStream_t)c.stream;
    const float *decay = c.decay;
    if (p.synth) {
        float *lg = (float *)(scr + l.logg);
        if (lasp::launch_fill_logg(p, c.decay, lg, stream) != hipSuccess) return LASP_ERR_HIP;
        decay = lg;
    }
    if (rebuild) {   // the forward pass's own plan (its segment count), states only, into the scratch tail
        lasp::Plan f;
        if (rc = make_plan(c.shape, kForward, &f, c.token, false); rc != LASP_OK) return rc;
        const lasp::FwdArgs fa{nullptr, c.k, c.v, c.kv_in, decay, nullptr, nullptr, (void *)cache, (float *)scr,
                               f.token ? (float *)(scr + l.seglog) : nullptr, nullptr, 0.0f, true};
        if (lasp::launch_fwd(f, fa, stream, nullptr) != hipSuccess) return LASP_ERR_HIP;
    }
    lasp::BwdArgs a{c.q, c.k, c.v, c.dout, c.dkv_out, decay, cache, c.dq, c.dk, c.dv, c.dkv_in, (float *)scr,
                    c.kv_out, c.dlog_g, p.token ? (float *)(scr + l.seglog) : nullptr,
                    p.token ? (float *)(scr + l.rtok) : nullptr, c.yn, c.rstd, nullptr, nullptr};
    if (p.kvdiv > 1) {   // the kernels write dK, dV per query head; launch_bwd sums each group into the outputs
        a.dk_out = c.dk;
        a.dv_out = c.dv;
        a.dk = scr + l.dk_part;
        a.dv = scr + l.dv_part;
    }
    return lasp::launch_bwd(p, a, stream, next_slot(1)) == hipSuccess ? LASP_OK : LASP_ERR_HIP;
}

// Bidirectional path: shape rules of the causal path, own K/V head per query head only.
int make_bidir_plan(const lasp_shape *s, lasp::BidirPlan *p) {
    if (!s) return LASP_ERR_NULL;
    if (s->dtype != LASP_F32 && s->dtype != LASP_BF16) return LASP_ERR_DTYPE;
    if (!valid_dims(s)) return LASP_ERR_SHAPE;
    if (s->kv_heads != 0 && s->kv_heads != s->H) return LASP_ERR_SHAPE;
    if (s->Dv != 0 && s->Dv != s->D) return LASP_ERR_SHAPE;
    p->B = s->B;
    p->H = s->H;
    p->N = s->N;
    p->D = s->D;
    p->dtype = s->dtype;
    const int tile = lasp::bidir_reduce_tile(s->dtype);
    p->ntiles_r = (s->N + tile - 1) / tile;
    int want = s->segments;
    if (want < 0 || want > p->ntiles_r) return LASP_ERR_SHAPE;
    if (want == 0) {
        const int64_t chains = (int64_t)s->B * s->H;
        want = (int)((lasp::kBidirTargetSegments + chains - 1) / chains);
        if (want > p->ntiles_r) want = p->ntiles_r;
    }
    p->tiles_per_seg = (p->ntiles_r + want - 1) / want;
    p->nseg = (p->ntiles_r + p->tiles_per_seg - 1) / p->tiles_per_seg;
    return LASP_OK;
}

size_t bidir_scratch(const lasp::BidirPlan &p) { return (size_t)p.B * p.H * p.nseg * p.D * p.D * sizeof(float); }

}  // namespace

namespace lasp {

hipError_t allow_dynamic_lds(const void *kernel, size_t bytes) {
    if (bytes <= 65536) return hipSuccess;
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    static std::mutex mu;
    static std::vector<std::pair<const void *, int>> raised;   // (kernel, device) pairs already set
    std::lock_guard<std::mutex> hold(mu);
    for (const auto &kd : raised)
        if (kd.first == kernel && kd.second == dev) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) raised.emplace_back(kernel, dev);
    return e;
}

}  // namespace lasp

extern "C" {

int lasp_version(void) { return 6; }

const char *lasp_status_str(int status) {
    switch (status) {
        case LASP_OK: return "ok";
        case LASP_ERR_NULL: return "a required pointer is NULL";
        case LASP_ERR_SHAPE: return "unsupported shape (need B,H,N > 0, D and Dv in {64,128} (Dv 0 = D), chunk in {64,128,256}, 0 <= segments <= ceil(N/tile))";
        case LASP_ERR_DTYPE: return "unsupported dtype (LASP_F32 or LASP_BF16)";
        case LASP_ERR_DECAY: return "decay must be finite and in (0, 1] (log decay: finite and <= 0)";
        case LASP_ERR_WORKSPACE: return "scratch buffer missing or too small (see lasp_scratch_bytes); lasp_fwd_noalloc: the shape needs more scratch than the library holds (see lasp_noalloc_scratch_limit)";
        case LASP_ERR_ALIAS: return "an output buffer overlaps an input or another output";
        case LASP_ERR_HIP: return "HIP runtime error at launch";
        case LASP_ERR_ALIGN: return "a buffer is not 16-byte aligned";
        default: return "unknown status";
    }
}

int lasp_check_shape(const lasp_shape *shape) {
    lasp::Plan p;
    return make_plan(shape, kForward, &p);
}

int lasp_check_decay(const float *decay_host, int32_t H) {
    if (!decay_host) return LASP_ERR_NULL;
    if (H <= 0) return LASP_ERR_SHAPE;
    for (int32_t h = 0; h < H; ++h) {
        float x = decay_host[h];
        if (!std::isfinite(x) || !(x > 0.0f) || x > 1.0f) return LASP_ERR_DECAY;
    }
    return LASP_OK;
}

int32_t lasp_tile_tokens(const lasp_shape *shape) {
    lasp::Plan p;
    return make_plan(shape, kForward, &p) == LASP_OK ? p.tile : 0;
}

int32_t lasp_num_segments(const lasp_shape *shape) {
    lasp::Plan p;
    return make_plan(shape, kForward, &p) == LASP_OK ? p.nseg : 0;
}

size_t lasp_state_cache_bytes(const lasp_shape *shape) { return cache_bytes(shape, false); }

size_t lasp_scratch_bytes(const lasp_shape *shape) {
    ScratchLayout l;
    return scratch_layout(shape, false, &l) ? l.total : 0;
}

size_t lasp_gated_state_cache_bytes(const lasp_shape *shape) { return cache_bytes(shape, true); }

size_t lasp_gated_scratch_bytes(const lasp_shape *shape) {
    ScratchLayout l;
    return scratch_layout(shape, true, &l) ? l.total : 0;
}

int lasp_check_log_decay(const float *log_g_host, int64_t n) {
    if (!log_g_host) return LASP_ERR_NULL;
    if (n <= 0) return LASP_ERR_SHAPE;
    for (int64_t i = 0; i < n; ++i) {
        float x = log_g_host[i];
        if (!std::isfinite(x) || x > 0.0f) return LASP_ERR_DECAY;
    }
    return LASP_OK;
}

int lasp_fwd(const lasp_shape *shape, const void *q, const void *k, const void *v, const float *kv_in,
             const float *decay, void *out, float *kv_out, void *state_cache, void *scratch,
             size_t scratch_bytes, void *hip_stream) {
    FwdCall c{shape, q, k, v, kv_in, decay, false, false, 0.0f, out, nullptr, kv_out, state_cache, scratch, scratch_bytes,
              hip_stream};
    return run_fwd_call(c);
}

int lasp_fwd_noalloc(const lasp_shape *shape, const void *q, const void *k, const void *v, const float *kv_in,
                     const float *decay, void *out, float *kv_out, void *state_cache, void *hip_stream) {
    ScratchLayout l;
    if (int rc = lasp_check_shape(shape); rc != LASP_OK) return rc;
    if (!scratch_layout(shape, false, &l)) return LASP_ERR_SHAPE;
    if (l.total > lasp::kStaticScratchBytes) return LASP_ERR_WORKSPACE;   // beyond the library's own scratch
    void *scr = nullptr;
    if (lasp::static_scratch(&scr) != hipSuccess) return LASP_ERR_HIP;
    FwdCall c{shape, q, k, v, kv_in, decay, false, false, 0.0f, out, nullptr, kv_out, state_cache, scr,
              lasp::kStaticScratchBytes, hip_stream};
    return run_fwd_call(c);
}

size_t lasp_noalloc_scratch_limit(void) { return lasp::kStaticScratchBytes; }

size_t lasp_bwd_recompute_scratch_bytes(const lasp_shape *shape) { return recompute_scratch(shape, false); }
size_t lasp_gated_bwd_recompute_scratch_bytes(const lasp_shape *shape) { return recompute_scratch(shape, true); }

int lasp_bwd(const lasp_shape *shape, const void *q, const void *k, const void *v, const void *dout,
             const float *kv_in, const float *dkv_out, const float *decay, const void *state_cache, void *dq, void *dk,
             void *dv, float *dkv_in, void *scratch, size_t scratch_bytes, void *hip_stream) {
    BwdCall c{shape, q, k, v, dout, kv_in, dkv_out, decay, false, false, nullptr, nullptr, nullptr, state_cache, dq, dk, dv,
              nullptr, dkv_in, scratch, scratch_bytes, hip_stream};
    return run_bwd_call(c);
}

int lasp_gated_fwd(const lasp_shape *shape, const void *q, const void *k, const void *v, const float *log_g,
                   const float *kv_in, void *out, float *kv_out, void *state_cache, void *scratch,
                   size_t scratch_bytes, void *hip_stream) {
    FwdCall c{shape, q, k, v, kv_in, log_g, true, false, 0.0f, out, nullptr, kv_out, state_cache, scratch, scratch_bytes,
              hip_stream};
    return run_fwd_call(c);
}

int lasp_gated_bwd(const lasp_shape *shape, const void *q, const void *k, const void *v, const void *dout,
                   const float *log_g, const float *kv_in, const float *kv_out, const float *dkv_out,
                   const void *state_cache, void *dq, void *dk, void *dv, float *dlog_g, float *dkv_in, void *scratch,
                   size_t scratch_bytes, void *hip_stream) {
    BwdCall c{shape, q, k, v, dout, kv_in, dkv_out, log_g, true, false, nullptr, nullptr, kv_out, state_cache, dq, dk, dv,
              dlog_g, dkv_in, scratch, scratch_bytes, hip_stream};
    return run_bwd_call(c);
}

int lasp_fwd_norm(const lasp_shape *shape, const void *q, const void *k, const void *v, const float *kv_in,
                  const float *decay, float eps, void *out, float *rstd, float *kv_out, void *state_cache,
                  void *scratch, size_t scratch_bytes, void *hip_stream) {
    FwdCall c{shape, q, k, v, kv_in, decay, false, true, eps, out, rstd, kv_out, state_cache, scratch, scratch_bytes,
              hip_stream};
    return run_fwd_call(c);
}

int lasp_bwd_norm(const lasp_shape *shape, const void *q, const void *k, const void *v, const void *out,
                  const float *rstd, const void *dout, const float *kv_in, const float *dkv_out, const float *decay,
                  const void *state_cache, void *dq, void *dk, void *dv, float *dkv_in, void *scratch,
                  size_t scratch_bytes, void *hip_stream) {
    BwdCall c{shape, q, k, v, dout, kv_in, dkv_out, decay, false, true, out, rstd, nullptr, state_cache, dq, dk, dv,
              nullptr, dkv_in, scratch, scratch_bytes, hip_stream};
    return run_bwd_call(c);
}

int lasp_gated_fwd_norm(const lasp_shape *shape, const void *q, const void *k, const void *v, const float *log_g,
                        const float *kv_in, float eps, void *out, float *rstd, float *kv_out, void *state_cache,
                        void *scratch, size_t scratch_bytes, void *hip_stream) {
    FwdCall c{shape, q, k, v, kv_in, log_g, true, true, eps, out, rstd, kv_out, state_cache, scratch, scratch_bytes,
              hip_stream};
    return run_fwd_call(c);
}

int lasp_gated_bwd_norm(const lasp_shape *shape, const void *q, const void *k, const void *v, const void *out,
                        const float *rstd, const void *dout, const float *log_g, const float *kv_in, const float *kv_out,
                        const float *dkv_out, const void *state_cache, void *dq, void *dk, void *dv,
                        float *dlog_g, float *dkv_in, void *scratch, size_t scratch_bytes, void *hip_stream) {
    BwdCall c{shape, q, k, v, dout, kv_in, dkv_out, log_g, true, true, out, rstd, kv_out, state_cache, dq, dk, dv,
              dlog_g, dkv_in, scratch, scratch_bytes, hip_stream};
    return run_bwd_call(c);
}

size_t lasp_bidir_scratch_bytes(const lasp_shape *shape) {
    lasp::BidirPlan p;
    return make_bidir_plan(shape, &p) == LASP_OK ? bidir_scratch(p) : 0;
}

int lasp_bidir_state(const lasp_shape *shape, const void *x, const void *y, float *state, int32_t accumulate,
                     void *scratch, size_t scratch_bytes, void *hip_stream) {
    lasp::BidirPlan p;
    int rc = make_bidir_plan(shape, &p);
    if (rc != LASP_OK) return rc;
    if (!x || !y || !state) return LASP_ERR_NULL;
    if (!scratch || scratch_bytes < bidir_scratch(p)) return LASP_ERR_WORKSPACE;
    const size_t tb = (size_t)p.B * p.H * p.N * p.D * elem_bytes(p.dtype);
    const size_t sb = (size_t)p.B * p.H * p.D * p.D * sizeof(float);
    rc = check_buffers({{x, tb}, {y, tb}}, {{state, sb}, {scratch, bidir_scratch(p)}});
    if (rc != LASP_OK) return rc;
    return lasp::launch_bidir_state(p, x, y, state, accumulate != 0, (float *)scratch, (hipStream_t)hip_stream,
                                    next_slot(0)) == hipSuccess ? LASP_OK : LASP_ERR_HIP;
}

int lasp_bidir_fwd(const lasp_shape *shape, const void *q, const float *kv, void *out, void *hip_stream) {
    lasp::BidirPlan p;
    int rc = make_bidir_plan(shape, &p);
    if (rc != LASP_OK) return rc;
    if (!q || !kv || !out) return LASP_ERR_NULL;
    const size_t tb = (size_t)p.B * p.H * p.N * p.D * elem_bytes(p.dtype);
    const size_t sb = (size_t)p.B * p.H * p.D * p.D * sizeof(float);
    rc = check_buffers({{q, tb}, {kv, sb}}, {{out, tb}});
    if (rc != LASP_OK) return rc;
    const lasp::BidirOps ops{{q, nullptr, nullptr}, {kv, nullptr, nullptr}, {out, nullptr, nullptr}, {0, 0, 0}};
    return lasp::launch_bidir_apply(p, ops, 1, (hipStream_t)hip_stream, next_slot(0)) == hipSuccess ? LASP_OK : LASP_ERR_HIP;
}

int lasp_bidir_bwd(const lasp_shape *shape, const void *k, const void *v, const void *dout, const float *kv,
                   const float *dkv, void *dq, void *dk, void *dv, void *hip_stream) {
    lasp::BidirPlan p;
    int rc = make_bidir_plan(shape, &p);
    if (rc != LASP_OK) return rc;
    if (!k || !v || !dout || !kv || !dkv || !dq || !dk || !dv) return LASP_ERR_NULL;
    const size_t tb = (size_t)p.B * p.H * p.N * p.D * elem_bytes(p.dtype);
    const size_t sb = (size_t)p.B * p.H * p.D * p.D * sizeof(float);
    rc = check_buffers({{k, tb}, {v, tb}, {dout, tb}, {kv, sb}, {dkv, sb}}, {{dq, tb}, {dk, tb}, {dv, tb}});
    if (rc != LASP_OK) return rc;
    // dQ = dO KV^T, dK = V dKV^T, dV = K dKV
    const lasp::BidirOps ops{{dout, v, k}, {kv, dkv, dkv}, {dq, dk, dv}, {1, 1, 0}};
    return lasp::launch_bidir_apply(p, ops, 3, (hipStream_t)hip_stream, next_slot(1)) == hipSuccess ? LASP_OK : LASP_ERR_HIP;
}

int lasp_profile_begin(int32_t max_calls) {
    if (max_calls <= 0 || g_prof.on) return LASP_ERR_SHAPE;
    for (int kind = 0; kind < 2; ++kind) {
        g_prof.slots[kind].assign(max_calls, lasp::KernelEvents{});
        for (auto &slot : g_prof.slots[kind])
            for (auto &ev : slot.ev)
                if (hipEventCreate(&ev) != hipSuccess) return LASP_ERR_HIP;
        g_prof.used[kind] = 0;
    }
    g_prof.cap = max_calls;
    g_prof.on = true;
    return LASP_OK;
}

int lasp_profile_end(double ms_sum[6], int32_t *fwd_calls, int32_t *bwd_calls) {
    if (!ms_sum || !fwd_calls || !bwd_calls) return LASP_ERR_NULL;
    if (!g_prof.on) return LASP_ERR_SHAPE;
    int rc = LASP_OK;
    for (int i = 0; i < 6; ++i) ms_sum[i] = 0.0;
    for (int kind = 0; kind < 2; ++kind) {
        for (int c = 0; c < g_prof.used[kind]; ++c) {
            const auto &slot = g_prof.slots[kind][c];
            if (hipEventSynchronize(slot.ev[3]) != hipSuccess) rc = LASP_ERR_HIP;
            for (int j = 0; j < 3; ++j) {
                float ms = 0.0f;
                if (hipEventElapsedTime(&ms, slot.ev[j], slot.ev[j + 1]) != hipSuccess) rc = LASP_ERR_HIP;
                ms_sum[3 * kind + j] += ms;
            }
        }
        for (auto &slot : g_prof.slots[kind])
            for (auto &ev : slot.ev) (void)hipEventDestroy(ev);
        g_prof.slots[kind].clear();
    }
    *fwd_calls = g_prof.used[0];
    *bwd_calls = g_prof.used[1];
    g_prof.on = false;
    g_prof.cap = 0;
    return rc;
}

}  // extern "C"
