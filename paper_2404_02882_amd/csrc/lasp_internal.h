// Internal interface between the C-ABI host layer (lasp_api.cpp) and the HIP
// kernels (lasp_kernels.hip). Not installed; the public boundary is include/lasp.h.
#ifndef LASP_INTERNAL_H
#define LASP_INTERNAL_H

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace lasp {

// Everything a launch needs, already validated by the host layer.
struct Plan {
    int B, H, N, D;     // D: the kernels' head dimension, max(dk, dv)
    int dk, dv;         // key (q, k) and value (v, out) dimensions as stored; the narrower one is zero-padded to D on chip
    int dtype;          // 0 = float, 1 = bfloat16
    int tile;           // tokens per kernel tile (CT)
    int ntiles;         // ceil(N / tile); only the last tile may be short, and only with token == true
    int nseg;           // segments per head (S)
    int tiles_per_seg;  // ceil(ntiles / nseg); the last segment may be shorter
    int cache_stride;   // the state cache holds the start state of every cache_stride-th tile (1 or 2)
    bool token;         // per-token decay: `decay` of the argument structs is log g, [B][H][N]
    bool norm;          // output rows are normalised (forward epilogue, backward prologue); token == false
    int kvdiv;          // query heads per K/V head (1 = every query head has its own)
    bool synth;         // one lambda per head but N % tile != 0: log g is synthesised and the token kernels run
};

struct FwdArgs {
    const void *q, *k, *v;
    const float *kv_in;   // may be null (zeros)
    const float *decay;   // lambda [H], or log g [B][H][N] with per-token decay
    void *out;
    float *kv_out;
    void *cache;          // may be null
    float *scratch;       // [B*H][nseg][D][D]
    float *seglog;        // per-token decay only: [B*H][nseg], log2 of the decay over each segment
    float *rstd_out;      // norm only: [B][H][N]
    float eps;            // norm only
    bool states_only;     // rebuild the state cache only: q, out, rstd_out are not touched (kv_out still is)
};

struct BwdArgs {
    const void *q, *k, *v, *dout;
    const float *dkv_out; // may be null (zeros)
    const float *decay;
    const void *cache;
    void *dq, *dk, *dv;
    float *dkv_in;
    float *scratch;
    // per-token decay only
    const float *kv_out;  // state the forward pass returned (needed when dkv_out is given)
    float *dlog_g;        // [B][H][N]
    float *seglog;        // [B*H][nseg]
    float *rtok;          // [B*H][N] scratch: q_t.dq_t - k_t.dk_t
    // norm only: `dout` is the gradient w.r.t. the normalised output
    const void *yn;       // the normalised output the forward pass wrote
    const float *rstd;    // [B][H][N], from the forward pass
    // grouped K/V heads only (kvdiv > 1): dk, dv above are per-query-head buffers in scratch,
    // summed over each group into these [B][kv_heads][N][D] outputs
    void *dk_out, *dv_out;
};

// Optional event recorder: when non-null, launch_* records ev[0] before the
// local pass, ev[1] after it, ev[2] after the scan and ev[3] after the walk.
struct KernelEvents {
    hipEvent_t ev[4];
};

// Raises the dynamic LDS limit of `kernel` (its host-side address) to `bytes` when that exceeds the 64 KB
// default. The attribute belongs to the kernel and the device's loaded module, so the runtime is asked
// once per (kernel, device) pair; later calls are a table lookup. Thread-safe.
hipError_t allow_dynamic_lds(const void *kernel, size_t bytes);

// The library's own scratch for lasp_fwd_noalloc: a file-scope device array of kStaticScratchBytes
// (32 MiB: 512 float [128][128] segment states, the automatic plan of 16 heads). static_scratch() returns
// its address on the current device (resolved once per device).
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
hipError_t static_scratch(void **ptr);

// Tile length used for a (dtype, chunk, D) combination.
int tile_tokens(int dtype, int chunk, int D);
// Cache stride for a shape: 2 (one cached state per pair of tiles, the backward
// walk reaches the other tile from its neighbour's state) when the kernels support it, else 1.
int cache_stride_for(int dtype, int tile, int ntiles, bool token, bool mixed_dims);

// log_g[b][h][s] = log(decay[h]) for all N tokens (device buffers).
hipError_t launch_fill_logg(const Plan &p, const float *decay, float *log_g, hipStream_t stream);
hipError_t launch_fwd(const Plan &p, const FwdArgs &a, hipStream_t stream, const KernelEvents *ke);
hipError_t launch_bwd(const Plan &p, const BwdArgs &a, hipStream_t stream, const KernelEvents *ke);


// Bidirectional (unmasked) path: O = Q (K^T V).
struct BidirPlan {
    int B, H, N, D, dtype;
    int ntiles_r;        // ceil(N / reduce tile)
    int nseg;            // segments per head of the state reduction (partial sums in scratch)
    int tiles_per_seg;   // ceil(ntiles_r / nseg); every segment non-empty
};
// Up to three products Out = X S (trans == 0) or X S^T (trans != 0), S [B*H][D][D] float.
struct BidirOps {
    const void *x[3];
    const float *s[3];
    void *out[3];
    int trans[3];
};
constexpr int kBidirTargetWorkgroups = 512;   // products: two 4-wave workgroups per CU
constexpr int kBidirTargetSegments = 256;     // reduction: one partial sum per CU (fewer partials to write and add)
int bidir_reduce_tile(int dtype);
// events: ev[0]..ev[1] the reduction, ev[1]..ev[2] the sum of the partials
hipError_t launch_bidir_state(const BidirPlan &p, const void *x, const void *y, float *state, int accumulate, float *part,
                              hipStream_t stream, const KernelEvents *ke);
// events: ev[2]..ev[3] the product kernel
hipError_t launch_bidir_apply(const BidirPlan &p, const BidirOps &ops, int nops, hipStream_t stream, const KernelEvents *ke);

}  // namespace lasp
#endif
