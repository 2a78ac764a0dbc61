// HIP kernels (gfx950 / CDNA4) for bidirectional (unmasked) linear attention,
// the right-product form O = Q (K^T V) of LASP (arxiv 2404.02882) Sec. 3.1,
// Eq. (3), without the Norm. There is no mask, no decay and no order among the
// tokens, so the path is two streaming passes:
//   k_bidir_reduce + k_bidir_sum : the d x d state, a plain sum over tokens,
//       state = sum_s x_s y_s^T (K^T V forward, Q^T dO backward). Every head is
//       cut into segments whose partial sums are added in a fixed order (no
//       atomics: results are bit-reproducible).
//   k_bidir_apply : Out = X S or X S^T for a d x d state held in registers,
//       forward O = Q KV; backward dQ = dO KV^T, dK = V dKV^T, dV = K dKV (the
//       three as one launch).
// Wave tiling and MFMA shapes as in lasp_kernels.hip: wave w owns the 32-wide
// column block w of the state and of every output tile.
#include <hip/hip_runtime.h>

#include "lasp_internal.h"
#include "lasp_device.h"

namespace lasp {

// ---------------------------------------------------------------------------
// k_bidir_reduce: partial state of one segment of one head,
//   part[chain][seg] = sum over the segment's tokens s of x_s y_s^T   ([a][c], a indexes x).
// Rows past the end of the sub-sequence read as zero.
// ---------------------------------------------------------------------------
template <typename T, int CT, int D>
__global__ __launch_bounds__(D * 2, 2) void k_bidir_reduce(const T *__restrict__ X, const T *__restrict__ Y,
                                                         float *__restrict__ part, int ntiles, int nseg,
                                                         int tiles_per_seg, int ntok) {
    using E = Elem<T>;
    constexpr int NT = D * 2, LDD = tile_ld<T, D>(), DB = D / 32, NKS = CT / E::KSTEP;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    T *sX = (T *)smem;
    T *sY = sX + CT * LDD;

    const int chain = blockIdx.y, seg = blockIdx.x;
    const int t0 = seg * tiles_per_seg;
    const int t1 = min(t0 + tiles_per_seg, ntiles);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave index, scalar
    Lane ln = fresh_lane();
    const size_t base = (size_t)chain * ntok * D;
    auto nvalid = [&](int t) { return min(CT, ntok - t * CT); };
    // Two tiles are in flight at any time: a streaming sum has nothing else to hide the memory latency with.
    TileMover<T, CT, D, NT, true> mx[2], my[2];   // streaming (non-temporal) loads
    auto request = [&](int b, int t) {
        if (t < t1) {
            mx[b].load(X + base + (size_t)t * CT * D, nvalid(t));
            my[b].load(Y + base + (size_t)t * CT * D, nvalid(t));
        }
    };
    request(0, t0);
    request(1, t0 + 1);
    f32x16 st[DB];
#pragma unroll
    for (int ab = 0; ab < DB; ++ab) st[ab] = f32x16{0};

    auto consume = [&](int b, int t) {
        __syncthreads();  // previous tile fully consumed
        ln = fresh_lane();
        mx[b].store(sX, LDD);
        my[b].store(sY, LDD);
        __syncthreads();
        request(b, t + 2);
        struct Step {
            typename E::frag y;
            typename E::frag x[DB];
        };
        pipelined<NKS>(
            [&](int ks) {
                Step f;
                f.y = E::ld_ks(ln, sY, LDD, ks * E::KSTEP, 32 * w);
#pragma unroll
                for (int ab = 0; ab < DB; ++ab) f.x[ab] = E::ld_ks(ln, sX, LDD, ks * E::KSTEP, 32 * ab);
                return f;
            },
            [&](int, const Step &f) {
#pragma unroll
                for (int ab = 0; ab < DB; ++ab) st[ab] = E::mfma(f.x[ab], f.y, st[ab]);
            });
    };
    for (int t = t0; t < t1; t += 2) {
        consume(0, t);
        if (t + 1 < t1) consume(1, t + 1);
    }
    state_store_w<D>(ln, st, part + ((size_t)chain * nseg + seg) * D * D, w);
}

// state[chain] = (accumulate ? state[chain] : 0) + part[chain][0] + part[chain][1] + ..., in that order.
__global__ __launch_bounds__(256) void k_bidir_sum(const float *__restrict__ part, float *__restrict__ state, int DD, int nseg,
                                                   int accumulate) {
    const int chain = blockIdx.y;
    const int e = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (e >= DD) return;
    float *dst = state + (size_t)chain * DD + e;
    const float *src = part + (size_t)chain * nseg * DD + e;
    f32x4 acc = accumulate ? *(const f32x4 *)dst : f32x4{0, 0, 0, 0};
    constexpr int U = 8;  // partial sums fetched together (independent loads)
    for (int n0 = 0; n0 < nseg; n0 += U) {
        f32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = n0 + u < nseg ? *(const f32x4 *)(src + (size_t)(n0 + u) * DD) : f32x4{0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u];
    }
    *(f32x4 *)dst = acc;
}

// ---------------------------------------------------------------------------
// k_bidir_apply: blockIdx.z selects one of up to three products Out = X S_eff,
// S_eff = S or S^T ([D][D] float per head, row-major). The wave's column block
// of S_eff is loaded once, converted to MFMA operand fragments, and kept in
// registers for every tile of the block's range:
//   OutT[c][i] = sum_a S_eff[a][c] X[i][a]      (a taken in accumulator order).
// ---------------------------------------------------------------------------
template <typename T, int CT, int D>
__global__ __launch_bounds__(D * 2, 2) void k_bidir_apply(BidirOps ops, int ntiles, int tiles_per_blk, int ntok) {
    using E = Elem<T>;
    constexpr int NT = D * 2, LDD = tile_ld<T, D>(), DB = D / 32, NB = CT / 32, LDO = D + 16 / (int)sizeof(T);
    extern __shared__ __attribute__((aligned(16))) char smem[];
    T *sX = (T *)smem;
    T *sO = sX + CT * LDD;   // output tile [token][feature], rows padded by 16 bytes

    const int chain = blockIdx.y, op = blockIdx.z;
    const int t0 = blockIdx.x * tiles_per_blk;
    const int t1 = min(t0 + tiles_per_blk, ntiles);
    if (t0 >= t1) return;  // uniform over the workgroup
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    Lane ln = fresh_lane();
    const size_t base = (size_t)chain * ntok * D;
    // uniform selects rather than indexing the by-value argument with a run-time index
    auto pick = [&](auto a, auto b, auto c) { return op == 0 ? a : op == 1 ? b : c; };
    const T *X = (const T *)pick(ops.x[0], ops.x[1], ops.x[2]) + base;
    T *O = (T *)pick(ops.out[0], ops.out[1], ops.out[2]) + base;
    const float *S = pick(ops.s[0], ops.s[1], ops.s[2]) + (size_t)chain * D * D;
    const int trans = pick(ops.trans[0], ops.trans[1], ops.trans[2]);
    auto nvalid = [&](int t) { return min(CT, ntok - t * CT); };
    // Two tiles are in flight at any time (nothing else hides the memory latency of a streaming product).
    TileMover<T, CT, D, NT> mx[2];
    auto request = [&](int b, int t) {
        if (t < t1) mx[b].load(X + (size_t)t * CT * D, nvalid(t));
    };
    request(0, t0);
    request(1, t0 + 1);

    typename E::frag sf[DB][E::NSUB];
    {
        f32x16 st[DB];
        if (trans) {
            // st[ab][i] = S[32 w + r][32 ab + acc_row(i)]: four consecutive floats per register group
            const unsigned lo = ((32 * w + ln.r) * D + 4 * ln.h) * sizeof(float);
#pragma unroll
            for (int ab = 0; ab < DB; ++ab)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v = gload<f32x4>(S + 32 * ab + 8 * g, lo);
#pragma unroll
                    for (int e = 0; e < 4; ++e) st[ab][4 * g + e] = v[e];
                }
        } else {
            state_load_w<D>(ln, st, S, w);
        }
#pragma unroll
        for (int ab = 0; ab < DB; ++ab)
#pragma unroll
            for (int m = 0; m < E::NSUB; ++m) sf[ab][m] = E::from_acc(st[ab], m);
    }

    auto consume = [&](int b, int t) {
        __syncthreads();  // previous tile fully consumed: sX and sO are free
        ln = fresh_lane();
        mx[b].store(sX, LDD);
        __syncthreads();
        request(b, t + 2);
        f32x16 acc[NB];
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) acc[ib] = f32x16{0};
#pragma unroll
        for (int ab = 0; ab < DB; ++ab)
#pragma unroll
            for (int m = 0; m < E::NSUB; ++m)
#pragma unroll
                for (int ib = 0; ib < NB; ++ib) acc[ib] = E::mfma(sf[ab][m], E::ld_kp(ln, sX, LDD, 32 * ib, 32 * ab, m), acc[ib]);
        // The accumulators hold the transposed tile (lane = token, four consecutive features per register
        // group). Written to memory as they are, a store instruction would touch 32 rows with 8 or 16 bytes
        // each; through LDS every row leaves as whole 16-byte pieces of consecutive lanes.
#pragma unroll
        for (int ib = 0; ib < NB; ++ib)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                E::st4(sO + (32 * ib + ln.r) * LDO + 32 * w + 8 * g + 4 * ln.h, acc[ib][4 * g], acc[ib][4 * g + 1],
                       acc[ib][4 * g + 2], acc[ib][4 * g + 3]);
        __syncthreads();
        {
            using M = TileMover<T, CT, D, NT>;
            const int row0 = threadIdx.x / M::VPR, nrows = nvalid(t);
            const unsigned glo = M::lane_off(D) * sizeof(T);
            const T *src = sO + M::lane_off(LDO);
            T *o = O + (size_t)t * CT * D;
#pragma unroll
            for (int i = 0; i < M::NV; ++i)
                if (row0 + i * (NT / M::VPR) < nrows)
                    gstore<u32x4>(o + i * (NT / M::VPR) * D, glo, *(const u32x4 *)(src + i * (NT / M::VPR) * LDO));
        }
    };
    for (int t = t0; t < t1; t += 2) {
        consume(0, t);
        if (t + 1 < t1) consume(1, t + 1);
    }
}

// ---------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------
template <typename T, int CT, int D>
static hipError_t run_bidir_state(const BidirPlan &p, const void *x, const void *y, float *state, int accumulate,
                                  float *part, hipStream_t s, const KernelEvents *ke) {
    const int chains = p.B * p.H, DD = D * D;
    constexpr size_t lds = 2 * (size_t)CT * tile_ld<T, D>() * sizeof(T);
    static_assert(lds <= 65536, "fits the default dynamic LDS limit");
    if (ke) (void)hipEventRecord(ke->ev[0], s);
    k_bidir_reduce<T, CT, D><<<dim3(p.nseg, chains), dim3(D * 2), lds, s>>>((const T *)x, (const T *)y, part, p.ntiles_r, p.nseg,
                                                                          p.tiles_per_seg, p.N);
    if (ke) (void)hipEventRecord(ke->ev[1], s);
    k_bidir_sum<<<dim3((DD / 4 + 255) / 256, chains), dim3(256), 0, s>>>(part, state, DD, p.nseg, accumulate);
    if (ke) {
        (void)hipEventRecord(ke->ev[2], s);
        (void)hipEventRecord(ke->ev[3], s);
    }
    return hipGetLastError();
}

template <typename T, int CT, int D>
static hipError_t run_bidir_apply(const BidirPlan &p, const BidirOps &ops, int nops, hipStream_t s, const KernelEvents *ke) {
    const int chains = p.B * p.H;
    constexpr size_t lds = (size_t)CT * (tile_ld<T, D>() + D + 16 / sizeof(T)) * sizeof(T);
    static_assert(2 * lds <= 163840, "two workgroups per CU");
    if (hipError_t e = allow_dynamic_lds((const void *)k_bidir_apply<T, CT, D>, lds); e != hipSuccess) return e;
    const int ntiles = (p.N + CT - 1) / CT;
    int nblk = (kBidirTargetWorkgroups + chains * nops - 1) / (chains * nops);
    if (nblk > ntiles) nblk = ntiles;
    const int tiles_per_blk = (ntiles + nblk - 1) / nblk;
    nblk = (ntiles + tiles_per_blk - 1) / tiles_per_blk;  // every block non-empty
    if (ke) {
        (void)hipEventRecord(ke->ev[0], s);
        (void)hipEventRecord(ke->ev[1], s);
        (void)hipEventRecord(ke->ev[2], s);
    }
    k_bidir_apply<T, CT, D><<<dim3(nblk, chains, nops), dim3(D * 2), lds, s>>>(ops, ntiles, tiles_per_blk, p.N);
    if (ke) (void)hipEventRecord(ke->ev[3], s);
    return hipGetLastError();
}

int bidir_reduce_tile(int dtype) { return dtype == 0 ? 32 : 64; }

hipError_t launch_bidir_state(const BidirPlan &p, const void *x, const void *y, float *state, int accumulate, float *part,
                              hipStream_t stream, const KernelEvents *ke) {
    if (p.dtype == 0) {
        if (p.D == 64) return run_bidir_state<float, 32, 64>(p, x, y, state, accumulate, part, stream, ke);
        return run_bidir_state<float, 32, 128>(p, x, y, state, accumulate, part, stream, ke);
    }
    if (p.D == 64) return run_bidir_state<bf16_t, 64, 64>(p, x, y, state, accumulate, part, stream, ke);
    return run_bidir_state<bf16_t, 64, 128>(p, x, y, state, accumulate, part, stream, ke);
}

// The apply pass keeps no state between tiles, so it reads long tiles: 128 tokens of bfloat16,
// 64 of float (more bytes in flight per workgroup, fewer barriers).
hipError_t launch_bidir_apply(const BidirPlan &p, const BidirOps &ops, int nops, hipStream_t stream, const KernelEvents *ke) {
    if (p.dtype == 0) {
        if (p.D == 64) return run_bidir_apply<float, 64, 64>(p, ops, nops, stream, ke);
        return run_bidir_apply<float, 64, 128>(p, ops, nops, stream, ke);
    }
    if (p.D == 64) return run_bidir_apply<bf16_t, 128, 64>(p, ops, nops, stream, ke);
    return run_bidir_apply<bf16_t, 128, 128>(p, ops, nops, stream, ke);
}

}  // namespace lasp
