// HIP kernels (gfx950 / CDNA4) for chunked causal linear attention with decay:
// the per-device hot path of LASP (arxiv 2404.02882, Alg. 2 forward, Alg. 3
// backward).
//
// Parallel structure. One head's sub-sequence is a serial recurrence over
// tiles, and there can be as few as 16 heads, so every head is cut into
// `nseg` segments of consecutive tiles that run as independent workgroups:
//   1. k_local : each segment accumulates its local state from zero
//                (forward: sum lambda^(len-s) k_s v_s^T; backward: sum
//                lambda^s q_s do_s^T), reading only K,V (or Q,dO).
//   2. k_scan  : an elementwise scan over the segments of a head turns the
//                local states into the state each segment starts from
//                (KV_t = lambda^len KV_{t-1} + local, the state update of
//                Sec. 3.2 taken over a whole segment).
//   3. k_fwd / k_bwd8p, k_bwd8, k_bwd : each segment walks its tiles with the
//                d x d state held in registers: intra-chunk left product,
//                inter-chunk right product, state update (Alg. 2 / Alg. 3 per
//                tile). Backward: k_bwd8p for bfloat16 with an even tile count
//                (one cached state per pair of tiles), k_bwd8 for an odd one,
//                k_bwd for float.
// Every kernel is instantiated for a decay model (lasp_device.h): one lambda
// per head, or a decay per token (general recurrent form of App. A.4), which
// adds k_dlg for the gradient of the log decay; optionally with the output
// normalisation fused (forward epilogue, backward prologue); and, where the key
// and value dimensions differ, for the row widths of the key-side and value-side
// tensors (the narrower rows are zero-padded on their way to LDS).
// This is the paper's "intra parts in parallel, inter parts in sequence"
// (Alg. 2) folded onto one GPU; there are no atomics, so results are
// bit-reproducible.
//
// Wave tiling. A workgroup has D/32 waves; wave w owns the 32-wide column block
// w of every [.][D] output tile and of the state, so the state tile it holds in
// MFMA accumulator layout can be fed back as the B operand of the next product
// without leaving registers (the contraction index is permuted identically on
// the A side). All products use 32x32 MFMA tiles: v_mfma_f32_32x32x16_bf16 for
// bfloat16 data, v_mfma_f32_32x32x2_f32 for float data; accumulation and the
// state are always fp32.
#include <hip/hip_runtime.h>

#include <mutex>

#include "lasp_internal.h"
#include "lasp_device.h"

namespace lasp {

// Grouped K/V heads: query heads h*kvdiv .. h*kvdiv+kvdiv-1 of a batch entry share K/V head h. The
// kernels index every token tensor by the query-head chain (b*H + h); K and V pointers are moved once,
// at kernel entry, by the distance between the chain's own slot and its K/V head's slot.
DEVI ptrdiff_t kv_shift(int chain, int H, int kvdiv, int ntok, int width) {
    const int kvchain = (chain / H) * (H / kvdiv) + (chain % H) / kvdiv;
    return (ptrdiff_t)(kvchain - chain) * ntok * width;
}
// First element of tile `t` (CT tokens) of a chain in a token tensor whose rows hold `width` elements.
DEVI size_t tile_off(int chain, int ntok, int t, int CT, int width) {
    return ((size_t)chain * ntok + (size_t)t * CT) * width;
}

// ---------------------------------------------------------------------------
// k_local: local state of a segment, from zero.
//   forward : local = sum_s lambda^(len - s) k_s v_s^T            (X = K, Y = V)
//   backward: local = sum_s lambda^s q_s do_s^T                    (X = Q, Y = dO)
// This is the state update of Alg. 2 / the dKV update of Alg. 3 unrolled over the segment's tiles: every
// token's weight is taken relative to the segment's edge (forward: its end, backward: its start) as
// (decay between the edge and the token's tile) x (the token's weight inside its tile), so the
// accumulators are plain sums and are never rescaled.
// The row weight is applied to the Y fragments (shared by all row blocks).
// ---------------------------------------------------------------------------
// NORM (backward only): Y is dY, the gradient w.r.t. the normalised output; the tile is turned into dO
// on its way to LDS from the normalised output `yn` and `rstd` ([chain][token]).
// WX, WY: elements per row of X and Y in memory (<= D; narrower rows are zero-padded on their way to LDS,
// which serves key and value dimensions that differ).
template <typename T, int CT, int D, bool BWD, bool TOKEN, bool NORM = false, int WX = D, int WY = D>
__global__ __launch_bounds__(D * 2, 2) void k_local(const T *__restrict__ X, const T *__restrict__ Y,
                                                  const float *__restrict__ decay, float *__restrict__ scratch,
                                                  float *__restrict__ seglog, int H, int ntiles, int nseg,
                                                  int tiles_per_seg, int ntok, int kvdiv, const T *__restrict__ yn = nullptr,
                                                  const float *__restrict__ rstd = nullptr) {
    static_assert(!NORM || BWD, "the Norm prologue belongs to the backward pass");
    using E = Elem<T>;
    constexpr int NT = D * 2, LDD = tile_ld<T, D>(), DB = D / 32, NKS = CT / E::KSTEP;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    T *sX = (T *)smem;
    T *sY = sX + CT * LDD;
    float *pw = (float *)(sY + CT * LDD);

    const int chain = blockIdx.y;
    const int seg = BWD ? blockIdx.x + 1 : blockIdx.x;
    const int t0 = seg * tiles_per_seg;
    const int t1 = min(t0 + tiles_per_seg, ntiles);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave index, scalar
    Lane ln = fresh_lane();
    if (!BWD) {  // forward: X, Y are K, V
        X += kv_shift(chain, H, kvdiv, ntok, WX);
        Y += kv_shift(chain, H, kvdiv, ntok, WY);
    }
    auto xoff = [&](int t) { return tile_off(chain, ntok, t, CT, WX); };
    auto yoff = [&](int t) { return tile_off(chain, ntok, t, CT, WY); };
    const int ntl = t1 - t0;
    auto tile_of = [&](int n) { return BWD ? t1 - 1 - n : t0 + n; };
    // the first tile is requested before anything else so that its latency covers the set-up
    // rows of tile `t` that exist: the last tile of a sub-sequence may be short (per-token decay only)
    auto nvalid = [&](int t) { return TOKEN ? min(CT, ntok - t * CT) : CT; };
    TileMover<T, CT, D, NT, true> mx, my;   // streaming (non-temporal) loads
    NormTile<T, CT, D, NT, WY> mn;   // the normalised output has the rows of Y (= dY)
    const float *rstd_c = rstd + (size_t)chain * ntok;
    if constexpr (!TOKEN) {   // (the per-token-decay path walks the tiles in the other order)
        mx.template load_w<WX>(X + xoff(tile_of(0)), nvalid(tile_of(0)));
        my.template load_w<WY>(Y + yoff(tile_of(0)), nvalid(tile_of(0)));
        if constexpr (NORM) mn.load(yn + yoff(tile_of(0)), rstd_c + (size_t)tile_of(0) * CT, nvalid(tile_of(0)));
    }
    f32x16 st[DB];
#pragma unroll
    for (int ab = 0; ab < DB; ++ab) st[ab] = f32x16{0};

    if constexpr (TOKEN) {
        // `decay` is log g, [chain][token]. The sum over the segment's tokens is taken walking AWAY from the
        // edge the weights refer to (forward: tiles descending from the segment's end, weight = decay over
        // the tokens after it; backward: tiles ascending from its start, weight = decay up to and including
        // it), so a token's weight is 2^(decay of the tiles already done + its weight inside its tile) and
        // the accumulators are never rescaled (same sum as the tile recursion of Alg. 2 / Alg. 3 unrolled).
        const TokenDecay<T, CT> dec(pw);
        const float *lg = decay + (size_t)chain * ntok;
        auto tile_at = [&](int n) { return BWD ? t0 + n : t1 - 1 - n; };
        mx.template load_w<WX>(X + xoff(tile_at(0)), nvalid(tile_at(0)));
        my.template load_w<WY>(Y + yoff(tile_at(0)), nvalid(tile_at(0)));
        if constexpr (NORM) mn.load(yn + yoff(tile_at(0)), rstd_c + (size_t)tile_at(0) * CT, nvalid(tile_at(0)));
        typename TokenDecay<T, CT>::LogG lgreg = TokenDecay<T, CT>::fetch(lg + (size_t)tile_at(0) * CT, nvalid(tile_at(0)));
        float base = 0.0f;   // log2 decay of the tiles already done (kept by the wave that fills the tables)
        for (int n = 0; n < ntl; ++n) {
            __syncthreads();
            ln = fresh_lane();
            if constexpr (NORM) mn.apply(my);
            mx.store(sX, LDD);
            my.store(sY, LDD);
            base += dec.fill(lgreg, base);
            __syncthreads();
            if (n + 1 < ntl) {
                const int tn = tile_at(n + 1);
                mx.template load_w<WX>(X + xoff(tn), nvalid(tn));
                my.template load_w<WY>(Y + yoff(tn), nvalid(tn));
                if constexpr (NORM) mn.load(yn + yoff(tn), rstd_c + (size_t)tn * CT, nvalid(tn));
                lgreg = TokenDecay<T, CT>::fetch(lg + (size_t)tn * CT, nvalid(tn));
            }
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
                [&](int ks, const Step &f) {
                    const typename E::frag yd = BWD ? dec.weigh_upto(ln, f.y, ks) : dec.weigh_after(ln, f.y, ks);
#pragma unroll
                    for (int ab = 0; ab < DB; ++ab) st[ab] = E::mfma(f.x[ab], yd, st[ab]);
                });
        }
        // log2 of the product of g over the segment, for the scan
        if (threadIdx.x == 0) seglog[(size_t)chain * nseg + seg] = base;
    } else {
    const float lam = decay[chain % H];
    fill_pow_table<CT>(pw, lam);
    const GeoWeights<T> geo(lam);
    const float l2f = (float)log2((double)lam);
    for (int n = 0; n < ntl; ++n) {
        __syncthreads();  // previous tile fully consumed (and pw visible on the first pass)
        ln = fresh_lane();
        if constexpr (NORM) mn.apply(my);
        mx.store(sX, LDD);
        my.store(sY, LDD);
        __syncthreads();
        if (n + 1 < ntl) {
            mx.template load_w<WX>(X + xoff(tile_of(n + 1)), CT);
            my.template load_w<WY>(Y + yoff(tile_of(n + 1)), CT);
            if constexpr (NORM) mn.load(yn + yoff(tile_of(n + 1)), rstd_c + (size_t)tile_of(n + 1) * CT);
        }
        // Token weight relative to the whole segment, so the accumulators are never rescaled:
        // forward lambda^(tokens after it in the segment), backward lambda^(its 1-based position).
        // It factors as (tile factor) * (table entry of the lane's first element) * g[e].
        const float tile_factor = exp2f((float)((ntl - 1 - n) * CT) * l2f);  // tiles between this one and the segment edge
        auto weight_of = [&](int ks) {
            const int k_first = ks * E::KSTEP + E::KH * ln.h;  // lane's first token of this fragment
            return tile_factor * (BWD ? pw[k_first + 1] : pw[CT - E::KH - k_first]);
        };
        if constexpr (NKS * (1 + DB) * sizeof(typename E::frag) <= 80 * 4) {
            // small tiles: request every operand fragment at once (one exposed LDS latency per tile)
            typename E::frag yf[NKS], xf[NKS][DB];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                yf[ks] = E::ld_ks(ln, sY, LDD, ks * E::KSTEP, 32 * w);
#pragma unroll
                for (int ab = 0; ab < DB; ++ab) xf[ks][ab] = E::ld_ks(ln, sX, LDD, ks * E::KSTEP, 32 * ab);
            }
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const typename E::frag yd = E::scale_geo(yf[ks], weight_of(ks), BWD ? geo.upto : geo.after);
#pragma unroll
                for (int ab = 0; ab < DB; ++ab) st[ab] = E::mfma(xf[ks][ab], yd, st[ab]);
            }
        } else {
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
                [&](int ks, const Step &f) {
                    const typename E::frag yd = E::scale_geo(f.y, weight_of(ks), BWD ? geo.upto : geo.after);
#pragma unroll
                    for (int ab = 0; ab < DB; ++ab) st[ab] = E::mfma(f.x[ab], yd, st[ab]);
                });
        }
    }
    }
    state_store_w<D, WX, WY>(ln, st, scratch + ((size_t)chain * nseg + seg) * WX * WY, w);
}

// ---------------------------------------------------------------------------
// k_scan: per state element, scan over the segments of a head.
//   forward : start_0 = kv_in (or 0); start_{j+1} = lambda^(len_j) start_j + local_j
//   backward: recv_{S-1} = dkv_out (or 0); recv_{j-1} = lambda^(len_j) recv_j + local_j
// scratch[chain][j] ([d_k][d_v] floats each) holds local_j on entry and start_j / recv_j on exit.
// ---------------------------------------------------------------------------
// With per-token decay the factor of segment j is 2^seglog[chain][j] (written by k_local).
template <bool BWD, bool TOKEN>
__global__ __launch_bounds__(256) void k_scan(float *__restrict__ scratch, const float *__restrict__ boundary,
                                              const float *__restrict__ decay, const float *__restrict__ seglog,
                                              int H, int DD, int nseg, int tiles_per_seg, int ntiles, int tile) {
    const int chain = blockIdx.y;
    const int e = (blockIdx.x * blockDim.x + threadIdx.x) * 4;  // four consecutive state elements per thread
    if (e >= DD) return;
    float p_full = 0.0f, p_last = 0.0f;
    if constexpr (!TOKEN) {
        const double l2 = log2((double)decay[chain % H]);
        p_full = (float)exp2((double)(tiles_per_seg * tile) * l2);
        p_last = (float)exp2((double)((ntiles - (nseg - 1) * tiles_per_seg) * tile) * l2);
    }
    // The caller's state and the segment states share one layout, [d_k][d_v] (DD = d_k * d_v elements).
    f32x4 carry = {0, 0, 0, 0};
    if (boundary) carry = *(const f32x4 *)(boundary + (size_t)chain * DD + e);
    float *s = scratch + (size_t)chain * nseg * DD + e;
    constexpr int U = 8;  // segments whose local states are fetched together (independent loads)
    for (int n0 = 0; n0 < nseg; n0 += U) {
        f32x4 local[U];
        float factor[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int n = n0 + u, j = BWD ? nseg - 1 - n : n;
            const bool has_local = n < nseg && (BWD ? (j > 0) : (j < nseg - 1));
            local[u] = has_local ? *(const f32x4 *)(s + (size_t)j * DD) : f32x4{0, 0, 0, 0};
            if constexpr (TOKEN) factor[u] = has_local ? exp2f(seglog[(size_t)chain * nseg + j]) : 0.0f;
            else factor[u] = j == nseg - 1 ? p_last : p_full;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int n = n0 + u, j = BWD ? nseg - 1 - n : n;
            if (n < nseg) {
                *(f32x4 *)(s + (size_t)j * DD) = carry;
                carry = factor[u] * carry + local[u];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// k_fwd: one segment of one head, tiles ascending (Alg. 2 per tile):
//   P      = (Q K^T) (.) M                       masked scores, via LDS
//   O      = P V + Lambda (Q KV_{t-1})           intra + inter
//   KV_t   = lambda^CT KV_{t-1} + (lambda^CT Lambda^-1 K)^T V
// The state KV_{t-1} each tile starts from is optionally written to the cache.
// ---------------------------------------------------------------------------
// NORM: every output row is divided by its root mean square (plus eps under the root) before it is
// stored, and the factor is written to rstd_out ([chain][token]) for the backward pass.
// WK, WV: elements per row of Q, K and of V, O in memory (<= D; see k_local).
// STATES: only the states are wanted (a backward pass that was given no state cache rebuilds it, Sec. 3.4's
// recomputation instead of caching): Q is not read, no scores and no outputs are computed; K, V are
// walked, every tile's entering state goes to the cache and the state is updated.
template <typename T, int CT, int D, bool TOKEN, bool NORM = false, int WK = D, int WV = D, bool STATES = false>
__global__ __launch_bounds__(D * 2, (CT <= 64 && sizeof(T) == 2) ? 2 : 1) void k_fwd(const T *__restrict__ Q, const T *__restrict__ K,
                                                const T *__restrict__ V, const float *__restrict__ decay,
                                                T *__restrict__ O, float *__restrict__ kv_out,
                                                T *__restrict__ cache, const float *__restrict__ scratch,
                                                int H, int ntiles, int nseg, int tiles_per_seg, int cache_stride, int ntok, int kvdiv,
                                                float *__restrict__ rstd_out = nullptr, float eps = 0.0f) {
    using E = Elem<T>;
    constexpr int NT = D * 2, LDD = tile_ld<T, D>(), LDP = CT + E::PAD, DB = D / 32, NB = CT / 32, NKS = CT / E::KSTEP,
                  SPB = 32 / E::KSTEP;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    T *sQ = (T *)smem;
    T *sK = sQ + CT * LDD;
    T *sV = sK + CT * LDD;
    T *sP = sV + CT * LDD;
    float *pw = (float *)(sP + CT * LDP);

    const int chain = blockIdx.y, seg = blockIdx.x;
    const int t0 = seg * tiles_per_seg;
    const int t1 = min(t0 + tiles_per_seg, ntiles);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave index, scalar
    Lane ln = fresh_lane();
    // requests first (tile, then start state), table arithmetic while they fly
    K += kv_shift(chain, H, kvdiv, ntok, WK);   // K, V of this chain's K/V head
    V += kv_shift(chain, H, kvdiv, ntok, WV);
    auto koff = [&](int t) { return tile_off(chain, ntok, t, CT, WK); };
    auto voff = [&](int t) { return tile_off(chain, ntok, t, CT, WV); };
    // rows of tile `t` that exist: the last tile of a sub-sequence may be short (per-token decay only)
    auto nvalid = [&](int t) { return TOKEN ? min(CT, ntok - t * CT) : CT; };
    static_assert(!STATES || !NORM, "the states do not depend on the Norm");
    TileMover<T, CT, D, NT> mq, mk, mv;
    if constexpr (!STATES) mq.template load_w<WK>(Q + koff(t0), nvalid(t0));
    mk.template load_w<WK>(K + koff(t0), nvalid(t0));
    mv.template load_w<WV>(V + voff(t0), nvalid(t0));
    f32x16 st[DB];
    state_load_w<D, WK, WV>(ln, st, scratch + ((size_t)chain * nseg + seg) * WK * WV, w);
    const auto dec = DecaySel<TOKEN, T, CT>::make(pw, decay, chain, H);
    const float *lg = decay + (size_t)chain * ntok;  // per-token decay: `decay` is log g, [chain][token]
    typename TokenDecay<T, CT>::LogG lgreg = {};
    if constexpr (TOKEN) lgreg = TokenDecay<T, CT>::fetch(lg + (size_t)t0 * CT, nvalid(t0));

    for (int t = t0; t < t1; ++t) {
        __syncthreads();
        ln = fresh_lane();
        // The state this tile starts from goes to the cache as KV_{t-1}, rows a, columns c.
        if (cache && t % cache_stride == 0)
            cache_store<T, CT, D, WK, WV>(ln, cache + ((size_t)chain * (ntiles / cache_stride) + t / cache_stride) * WK * WV, st, sP, w);
        if constexpr (!STATES) mq.store(sQ, LDD);
        mk.store(sK, LDD);
        mv.store(sV, LDD);
        if constexpr (TOKEN) dec.fill(lgreg);
        __syncthreads();
        if (t + 1 < t1) {
            if constexpr (!STATES) mq.template load_w<WK>(Q + koff(t + 1), nvalid(t + 1));
            mk.template load_w<WK>(K + koff(t + 1), nvalid(t + 1));
            mv.template load_w<WV>(V + voff(t + 1), nvalid(t + 1));
            if constexpr (TOKEN) lgreg = TokenDecay<T, CT>::fetch(lg + (size_t)(t + 1) * CT, nvalid(t + 1));
        }
        if constexpr (!STATES) {
        // masked scores P (all waves share the lower-triangular blocks)
        masked_scores<T, CT, D, LDD, LDP>(ln, sP, sK, sQ, dec, w);

        __syncthreads();  // P visible
        ln = fresh_lane();

        // Output tiles are accumulated transposed: OT[c][i], c in this wave's column block.
        f32x16 acc[NB];
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) acc[ib] = f32x16{0};
        // inter: OT[c][i] = sum_a KV_{t-1}[a][c] Q[i][a], a taken in accumulator order
#pragma unroll
        for (int ab = 0; ab < DB; ++ab)
#pragma unroll
            for (int m = 0; m < E::NSUB; ++m) {
                const typename E::frag sf = E::from_acc(st[ab], m);
#pragma unroll
                for (int ib = 0; ib < NB; ++ib) acc[ib] = E::mfma(sf, E::ld_kp(ln, sQ, LDD, 32 * ib, 32 * ab, m), acc[ib]);
            }
        // Lambda: token r (1-based) carries lambda^r; the token is this lane's column
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) acc[ib] *= dec.upto(32 * ib + ln.r);
        // intra: OT[c][i] += sum_{j<=i} V[j][c] P[i][j]
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const typename E::frag vf = E::ld_ks(ln, sV, LDD, ks * E::KSTEP, 32 * w);
#pragma unroll
            for (int ib = ks / SPB; ib < NB; ++ib) acc[ib] = E::mfma(vf, E::ld_kc(ln, sP, LDP, 32 * ib, ks * E::KSTEP), acc[ib]);
        }
        if constexpr (NORM) {
            // sum of squares of a token's row: this wave's 32 features, then the other waves' through LDS
            float *red = pw + 3 * CT + 4;
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
                float ss = 0.0f;
#pragma unroll
                for (int i = 0; i < 16; ++i) ss += acc[ib][i] * acc[ib][i];
                ss = add_other_half(ss);
                if (ln.h == 0) red[w * CT + 32 * ib + ln.r] = ss;
            }
            __syncthreads();
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
                float tot = 0.0f;
#pragma unroll
                for (int wv = 0; wv < D / 32; ++wv) tot += red[wv * CT + 32 * ib + ln.r];
                const float rs = rsqrtf(tot * (1.0f / WV) + eps);   // mean over the real value features (padding is zero)
                acc[ib] *= rs;
                if (w == 0 && ln.h == 0 && 32 * ib + ln.r < nvalid(t))
                    rstd_out[(size_t)chain * ntok + (size_t)t * CT + 32 * ib + ln.r] = rs;
            }
        }
        T *o = O + voff(t);
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) store_out_tile_t<T, D, WV>(ln, o, acc[ib], 32 * ib, w, nvalid(t));
        }   // !STATES

        ln = fresh_lane();
        // state update: KV <- lambda^CT KV + (diag{lambda^(CT-1-j)} K)^T V, weight applied to the V fragments
        const float lamC = dec.whole();
#pragma unroll
        for (int ab = 0; ab < DB; ++ab) st[ab] *= lamC;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const typename E::frag vd = dec.weigh_after(ln, E::ld_ks(ln, sV, LDD, ks * E::KSTEP, 32 * w), ks);
#pragma unroll
            for (int ab = 0; ab < DB; ++ab) st[ab] = E::mfma(E::ld_ks(ln, sK, LDD, ks * E::KSTEP, 32 * ab), vd, st[ab]);
        }
    }
    if (seg == nseg - 1 && kv_out) state_store_w<D, WK, WV>(ln, st, kv_out + (size_t)chain * WK * WV, w);
}

// ---------------------------------------------------------------------------
// k_bwd: one segment of one head, tiles descending (Alg. 3 per tile):
//   dSm = (dO V^T) (.) M,  Sm = (Q K^T) (.) M
//   dQ  = dSm K + Lambda (dO KV_{t-1}^T)
//   dK  = dSm^T Q + (lambda^CT Lambda^-1) (V dKV^T)
//   dV  = Sm^T dO + (lambda^CT Lambda^-1) (K dKV)
//   dKV <- lambda^CT dKV + (Lambda Q)^T dO
// dKV is the state received from the right (gradient w.r.t. KV_t). The wave
// keeps its column block dKV[:, c in w] in registers, which serves dV directly;
// dK needs the transposed block, fetched once per tile through an LDS exchange.
// LDS is time-shared: first {V, dO}, then {K, Q}.
// ---------------------------------------------------------------------------
template <typename T, int CT, int D>
struct BwdSmem {
    using E = Elem<T>;
    static constexpr int LDD = tile_ld<T, D>(), LDP = CT + E::PAD;
    static constexpr size_t IN_BYTES = 2 * (size_t)CT * LDD * sizeof(T);   // two input tiles
    static constexpr size_t X_BYTES = (size_t)D * LDD * sizeof(T);         // exchange buffer
    static constexpr bool OVERLAY = X_BYTES <= IN_BYTES;                    // exchange reuses the input tiles
    static constexpr size_t P_OFF = IN_BYTES + (OVERLAY ? 0 : X_BYTES);
    static constexpr size_t PW_OFF = P_OFF + 2 * (size_t)CT * LDP * sizeof(T);
    static constexpr size_t TOTAL = PW_OFF + table_floats<CT>() * sizeof(float);
};

// NORM: dO is dY, the gradient w.r.t. the normalised output `yn`; every dY tile is turned into dO on its
// way to LDS (NormTile) from `yn` and `rstd` ([chain][token]).
// WK, WV: elements per row of Q, K, dQ, dK and of V, dO, dV in memory (<= D; see k_local).
template <typename T, int CT, int D, bool TOKEN, bool NORM = false, int WK = D, int WV = D>
__global__ __launch_bounds__(D * 2, (CT <= 64 && sizeof(T) == 2 && WK == D && WV == D) ? 2 : 1) void k_bwd(const T *__restrict__ Q, const T *__restrict__ K,
                                                const T *__restrict__ V, const T *__restrict__ dO,
                                                const float *__restrict__ decay, const T *__restrict__ cache,
                                                T *__restrict__ dQ, T *__restrict__ dK, T *__restrict__ dV,
                                                float *__restrict__ dkv_in, const float *__restrict__ scratch,
                                                float *__restrict__ rtok,
                                                int H, int ntiles, int nseg, int tiles_per_seg, int ntok, int kvdiv,
                                                const T *__restrict__ yn = nullptr, const float *__restrict__ rstd = nullptr) {
    using E = Elem<T>;
    using SM = BwdSmem<T, CT, D>;
    constexpr int NT = D * 2, LDD = SM::LDD, LDP = SM::LDP, DB = D / 32, NB = CT / 32, NKS = CT / E::KSTEP,
                  NKD = D / E::KSTEP, SPB = 32 / E::KSTEP;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    T *bufA = (T *)smem;
    T *bufB = bufA + CT * LDD;
    T *sX = SM::OVERLAY ? bufA : (T *)(smem + SM::IN_BYTES);
    T *sS = (T *)(smem + SM::P_OFF);
    T *sDS = sS + CT * LDP;
    float *pw = (float *)(smem + SM::PW_OFF);

    const int chain = blockIdx.y, seg = blockIdx.x;
    const int t0 = seg * tiles_per_seg;
    const int t1 = min(t0 + tiles_per_seg, ntiles);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave index, scalar
    Lane ln = fresh_lane();
    const auto dec = DecaySel<TOKEN, T, CT>::make(pw, decay, chain, H);
    const float *lg = decay + (size_t)chain * ntok;  // per-token decay: `decay` is log g, [chain][token]
    typename TokenDecay<T, CT>::LogG lgreg = {};
    // rows of tile `t` that exist: the last tile of a sub-sequence may be short (per-token decay only)
    auto nvalid = [&](int t) { return TOKEN ? min(CT, ntok - t * CT) : CT; };
    if constexpr (TOKEN) lgreg = TokenDecay<T, CT>::fetch(lg + (size_t)(t1 - 1) * CT, nvalid(t1 - 1));
    // per-token decay: r_t = q_t.dq_t - k_t.dk_t, one partial row per wave, summed and written per tile
    float *rs = pw + 3 * CT + 4;
    auto flush_r = [&](int tile) {
        if (threadIdx.x < CT) {
            float r = 0.0f;
#pragma unroll
            for (int wv = 0; wv < D / 32; ++wv) r += rs[wv * CT + threadIdx.x];
            if (tile * CT + (int)threadIdx.x < ntok) rtok[(size_t)chain * ntok + (size_t)tile * CT + threadIdx.x] = r;
        }
    };

    K += kv_shift(chain, H, kvdiv, ntok, WK);   // K, V of this chain's K/V head
    V += kv_shift(chain, H, kvdiv, ntok, WV);
    auto koff = [&](int t) { return tile_off(chain, ntok, t, CT, WK); };
    auto voff = [&](int t) { return tile_off(chain, ntok, t, CT, WV); };
    f32x16 dkv[DB];
    state_load_w<D, WK, WV>(ln, dkv, scratch + ((size_t)chain * nseg + seg) * WK * WV, w);

    TileMover<T, CT, D, NT> ma, mb;
    ma.template load_w<WV>(V + voff(t1 - 1), nvalid(t1 - 1));
    mb.template load_w<WV>(dO + voff(t1 - 1), nvalid(t1 - 1));
    NormTile<T, CT, D, NT, WV> mn;
    const float *rstd_c = rstd + (size_t)chain * ntok;
    if constexpr (NORM) mn.load(yn + voff(t1 - 1), rstd_c + (size_t)(t1 - 1) * CT, nvalid(t1 - 1));

    for (int t = t1 - 1; t >= t0; --t) {
        // ---- exchange: dKV^T fragments for dK_inter (B[k = c][n = a in w]) ----
        __syncthreads();
        ln = fresh_lane();
        if constexpr (TOKEN) {
            if (t < t1 - 1) flush_r(t + 1);
        }
#pragma unroll
        for (int ab = 0; ab < DB; ++ab)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                E::st4(sX + lds_off(LDD, 32 * w + ln.r, 32 * ab + 8 * g + 4 * ln.h), dkv[ab][4 * g], dkv[ab][4 * g + 1],
                       dkv[ab][4 * g + 2], dkv[ab][4 * g + 3]);
        __syncthreads();
        typename E::frag xf[NKD];
#pragma unroll
        for (int ks = 0; ks < NKD; ++ks) xf[ks] = E::ld_ks(ln, sX, LDD, ks * E::KSTEP, 32 * w);
        __syncthreads();

        // ---- step 1: V (bufA), dO (bufB) ----
        if constexpr (NORM) mn.apply(mb);
        ma.store(bufA, LDD);
        mb.store(bufB, LDD);
        if constexpr (TOKEN) dec.fill(lgreg);
        __syncthreads();
        ma.template load_w<WK>(K + koff(t), nvalid(t));
        mb.template load_w<WK>(Q + koff(t), nvalid(t));
        if constexpr (TOKEN) {
            if (t > t0) lgreg = TokenDecay<T, CT>::fetch(lg + (size_t)(t - 1) * CT);   // only the last tile can be short
        }

        masked_scores<T, CT, D, LDD, LDP>(ln, sDS, bufA, bufB, dec, w);  // dS^T = V dO^T

        // All output tiles are accumulated transposed (feature x token), this wave's feature block.
        f32x16 accQ[NB], accK[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) accQ[b] = accK[b] = f32x16{0};
        // dQ_inter^T[a][i] = lambda^i sum_c KV_{t-1}[a][c] dO[i][c]; KV rows are read from the cache in place
        {
            const T *c = cache + ((size_t)chain * ntiles + t) * WK * WV;   // [WK][WV]: rows and columns of padding are not there
#pragma unroll
            for (int ks = 0; ks < NKD; ++ks) {
                typename E::frag kvf = {};
                if (32 * w < WK && ks * E::KSTEP < WV) kvf = E::ld_kc_g(ln, c, WV, 32 * w, ks * E::KSTEP);
#pragma unroll
                for (int ib = 0; ib < NB; ++ib) accQ[ib] = E::mfma(kvf, E::ld_kc(ln, bufB, LDD, 32 * ib, ks * E::KSTEP), accQ[ib]);
            }
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) accQ[ib] *= dec.upto(32 * ib + ln.r);
        }
        // dK_inter^T[a][j] = lambda^(CT-j) sum_c dKV[a][c] V[j][c]
#pragma unroll
        for (int ks = 0; ks < NKD; ++ks)
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) accK[jb] = E::mfma(xf[ks], E::ld_kc(ln, bufA, LDD, 32 * jb, ks * E::KSTEP), accK[jb]);
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) accK[jb] *= dec.after(32 * jb + ln.r);
        // dO fragments of this wave's column block: [k = i][n = c in w]
        typename E::frag dof[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) dof[ks] = E::ld_ks(ln, bufB, LDD, ks * E::KSTEP, 32 * w);

        // ---- step 2: K (bufA), Q (bufB) ----
        __syncthreads();
        ln = fresh_lane();
        ma.store(bufA, LDD);
        mb.store(bufB, LDD);
        __syncthreads();
        if (t > t0) {
            ma.template load_w<WV>(V + voff(t - 1), CT);
            mb.template load_w<WV>(dO + voff(t - 1), CT);
            if constexpr (NORM) mn.load(yn + voff(t - 1), rstd_c + (size_t)(t - 1) * CT);
        }
        masked_scores<T, CT, D, LDD, LDP>(ln, sS, bufA, bufB, dec, w);  // S^T = K Q^T
        __syncthreads();

        // dQ^T[a][i] += sum_{j<=i} K[j][a] dSm[i][j]
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const typename E::frag kf = E::ld_ks(ln, bufA, LDD, ks * E::KSTEP, 32 * w);
#pragma unroll
            for (int ib = ks / SPB; ib < NB; ++ib) accQ[ib] = E::mfma(kf, E::ld_kc(ln, sDS, LDP, 32 * ib, ks * E::KSTEP), accQ[ib]);
        }
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) store_out_tile_t<T, D, WK>(ln, dQ + koff(t), accQ[ib], 32 * ib, w, nvalid(t));
        float rpart[NB];
        if constexpr (TOKEN) {
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) rpart[ib] = rowdot<T>(ln, accQ[ib], bufB, LDD, 32 * ib, w);
        }
        // dK^T[a][j] += sum_{i>=j} Q[i][a] dSm[i][j]
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const typename E::frag qf = E::ld_ks(ln, bufB, LDD, ks * E::KSTEP, 32 * w);
#pragma unroll
            for (int jb = 0; jb <= ks / SPB; ++jb) accK[jb] = E::mfma(qf, E::ld_ks(ln, sDS, LDP, ks * E::KSTEP, 32 * jb), accK[jb]);
        }
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) store_out_tile_t<T, D, WK>(ln, dK + koff(t), accK[jb], 32 * jb, w, nvalid(t));
        if constexpr (TOKEN) {
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                rpart[jb] -= rowdot<T>(ln, accK[jb], bufA, LDD, 32 * jb, w);
                if (ln.h == 0) rs[w * CT + 32 * jb + ln.r] = rpart[jb];
            }
        }
        // dV^T[c][j] = lambda^(CT-j) sum_a dKV[a][c] K[j][a] + sum_{i>=j} dO[i][c] Sm[i][j]
        {
            f32x16 accV[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) accV[jb] = f32x16{0};
#pragma unroll
            for (int ab = 0; ab < DB; ++ab)
#pragma unroll
                for (int m = 0; m < E::NSUB; ++m) {
                    const typename E::frag df = E::from_acc(dkv[ab], m);
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb) accV[jb] = E::mfma(df, E::ld_kp(ln, bufA, LDD, 32 * jb, 32 * ab, m), accV[jb]);
                }
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) accV[jb] *= dec.after(32 * jb + ln.r);
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                for (int jb = 0; jb <= ks / SPB; ++jb)
                    accV[jb] = E::mfma(dof[ks], E::ld_ks(ln, sS, LDP, ks * E::KSTEP, 32 * jb), accV[jb]);
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) store_out_tile_t<T, D, WV>(ln, dV + voff(t), accV[jb], 32 * jb, w, nvalid(t));
        }
        // dKV <- lambda^CT dKV + (Lambda Q)^T dO  (row weight lambda^(i+1) applied to the dO fragments)
        const float lamC = dec.whole();
#pragma unroll
        for (int ab = 0; ab < DB; ++ab) dkv[ab] *= lamC;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const typename E::frag dos = dec.weigh_upto(ln, dof[ks], ks);
#pragma unroll
            for (int ab = 0; ab < DB; ++ab) dkv[ab] = E::mfma(E::ld_ks(ln, bufB, LDD, ks * E::KSTEP, 32 * ab), dos, dkv[ab]);
        }
    }
    if constexpr (TOKEN) {
        __syncthreads();
        flush_r(t0);
    }
    if (seg == 0) state_store_w<D, WK, WV>(ln, dkv, dkv_in + (size_t)chain * WK * WV, w);
}

// ---------------------------------------------------------------------------
// k_bwd8: the backward walk for bfloat16 tiles of 64 tokens, one workgroup of
// 2 * D/32 waves per CU. Same mathematics as k_bwd, different residency:
//   - all four input tiles (V, dO, K, Q), both masked score tiles and the
//     cached KV_{t-1} tile live in LDS at once, so a tile needs three barriers;
//   - the waves form two groups that each keep dKV in registers in the
//     orientation their product needs, so nothing is exchanged:
//       group 0 holds dKV[a][c in w] (rows a) and produces dV (dV_inter contracts a),
//       group 1 holds dKV[a in w][c] (rows c) and produces dK (dK_inter contracts c);
//     under the exchange K<->V, Q<->dO, S<->dS the two products are the same
//     code, including the dKV update, so the groups differ only in pointers;
//   - dQ needs only the cached state and is split by token block between them
//     (group 0, which the hardware favours when both wait to issue, takes the
//     block with the longer key range).
// ---------------------------------------------------------------------------
template <typename T, int CT, int D>
struct Bwd8Smem {
    using E = Elem<T>;
    static constexpr int LDD = tile_ld<T, D>(), LDP = CT + E::PAD;
    static constexpr size_t TILE = (size_t)CT * LDD * sizeof(T);
    static constexpr size_t P_OFF = 4 * TILE;
    static constexpr size_t C_OFF = P_OFF + 2 * (size_t)CT * LDP * sizeof(T);   // cached KV_{t-1} tile
    static constexpr size_t PW_OFF = C_OFF + (size_t)D * LDD * sizeof(T);
    static constexpr size_t TOTAL = PW_OFF + table_floats<CT>() * sizeof(float);
};

template <typename T, int CT, int D, bool TOKEN, bool NORM = false>
__global__ __launch_bounds__(D * 4) void k_bwd8(const T *__restrict__ Q, const T *__restrict__ K,
                                                 const T *__restrict__ V, const T *__restrict__ dO,
                                                 const float *__restrict__ decay, const T *__restrict__ cache,
                                                 T *__restrict__ dQ, T *__restrict__ dK, T *__restrict__ dV,
                                                 float *__restrict__ dkv_in, const float *__restrict__ scratch,
                                                 float *__restrict__ rtok,
                                                 int H, int ntiles, int nseg, int tiles_per_seg, int ntok, int kvdiv,
                                                 const T *__restrict__ yn = nullptr, const float *__restrict__ rstd = nullptr) {
    using E = Elem<T>;
    using F = typename E::frag;
    using SM = Bwd8Smem<T, CT, D>;
    static_assert(CT == 64, "two 32-token blocks per tile");
    constexpr int NT = D * 4, NW = D / 32, LDD = SM::LDD, LDP = SM::LDP, DB = D / 32, NB = CT / 32, NKS = CT / E::KSTEP,
                  NKD = D / E::KSTEP, SPB = 32 / E::KSTEP;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    T *sV = (T *)smem;
    T *sdO = sV + CT * LDD;
    T *sK = sdO + CT * LDD;
    T *sQ = sK + CT * LDD;
    T *sS = (T *)(smem + SM::P_OFF);
    T *sDS = sS + CT * LDP;
    T *sC = (T *)(smem + SM::C_OFF);
    float *pw = (float *)(smem + SM::PW_OFF);

    const int chain = blockIdx.y, seg = blockIdx.x;
    const int t0 = seg * tiles_per_seg;
    const int t1 = min(t0 + tiles_per_seg, ntiles);
    const int w8 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int w = w8 % NW;    // feature block of this wave's outputs
    const int rg = w8 / NW;   // group: 0 produces dV, 1 produces dK
    Lane ln = fresh_lane();

    // requests first (last tile of the segment, its cached state), set-up arithmetic while they fly
    const size_t base = (size_t)chain * ntok * D;
    {   // K, V of this chain's K/V head
        const ptrdiff_t sh = kv_shift(chain, H, kvdiv, ntok, D);
        K += sh;
        V += sh;
    }
    TileMover<T, CT, D, NT> mv, mo, mk, mq;
    TileMover<T, D, D, NT> mc;  // cached state tile KV_{t-1}, [a][c]
    const T *ctile = cache + (size_t)chain * ntiles * D * D;
    {
        const size_t off = base + (size_t)(t1 - 1) * CT * D;
        const int nv = TOKEN ? min(CT, ntok - (t1 - 1) * CT) : CT;  // the last tile of a sub-sequence may be short
        mv.load(V + off, nv);
        mo.load(dO + off, nv);
        mk.load(K + off, nv);
        mq.load(Q + off, nv);
        mc.load(ctile + (size_t)(t1 - 1) * D * D);
    }
    NormTile<T, CT, D, NT> mn;  // NORM: dO is dY; turned into dO from the normalised output and rstd on its way to LDS
    const float *rstd_c = rstd + (size_t)chain * ntok;
    if constexpr (NORM)
        mn.load(yn + base + (size_t)(t1 - 1) * CT * D, rstd_c + (size_t)(t1 - 1) * CT, TOKEN ? min(CT, ntok - (t1 - 1) * CT) : CT);
    const auto dec = DecaySel<TOKEN, T, CT>::make(pw, decay, chain, H);
    const float *lg = decay + (size_t)chain * ntok;  // per-token decay: `decay` is log g, [chain][token]
    typename TokenDecay<T, CT>::LogG lgreg = {};
    if constexpr (TOKEN) lgreg = TokenDecay<T, CT>::fetch(lg + (size_t)(t1 - 1) * CT, min(CT, ntok - (t1 - 1) * CT));
    // per-token decay: r_t = q_t.dq_t - k_t.dk_t, one partial row per wave, summed and written per tile
    float *rs = pw + 3 * CT + 4;
    auto flush_r = [&](int tile) {
        if (threadIdx.x < CT) {
            float r = 0.0f;
#pragma unroll
            for (int wv = 0; wv < 2 * NW; ++wv) r += rs[wv * CT + threadIdx.x];
            if (tile * CT + (int)threadIdx.x < ntok) rtok[(size_t)chain * ntok + (size_t)tile * CT + threadIdx.x] = r;
        }
    };

    // Group-dependent operands (wave-uniform selects).
    const T *sX1 = rg ? sV : sK;     // inter operand: token rows, features contracted with the state
    const T *sX2 = rg ? sQ : sdO;    // intra operand and state-update B operand: [token][feature in w]
    const T *sUA = rg ? sdO : sQ;    // state-update A operand: [token][feature of the state rows]
    const T *sPm = rg ? sDS : sS;    // masked score tile P[i][j] of this product
    T *gOut = rg ? dK : dV;

    // st[blk][i]: group 0: dKV[32 blk + acc_row(i)][32 w + r]; group 1: dKV[32 w + r][32 blk + acc_row(i)]
    f32x16 st[DB];
    {
        const float *g = scratch + ((size_t)chain * nseg + seg) * D * D;
        if (rg == 0) state_load_w<D>(ln, st, g, w);
        else state_load_t_w<D>(ln, st, g, w);
    }

    for (int t = t1 - 1; t >= t0; --t) {
        const size_t off = base + (size_t)t * CT * D;
        const int nrows = TOKEN ? min(CT, ntok - t * CT) : CT;  // rows of this tile that exist
        __syncthreads();  // previous tile fully consumed
        ln = fresh_lane();
        if constexpr (TOKEN) {
            if (t < t1 - 1) flush_r(t + 1);
            dec.fill(lgreg);
        }
        if constexpr (NORM) mn.apply(mo);
        mv.store(sV, LDD);
        mo.store(sdO, LDD);
        mk.store(sK, LDD);
        mq.store(sQ, LDD);
        mc.store(sC, LDD);
        __syncthreads();
        ln = fresh_lane();
        if (t > t0) {
            mv.load(V + off - (size_t)CT * D);
            mo.load(dO + off - (size_t)CT * D);
            mk.load(K + off - (size_t)CT * D);
            mq.load(Q + off - (size_t)CT * D);
            mc.load(ctile + (size_t)(t - 1) * D * D);
            if constexpr (NORM) mn.load(yn + off - (size_t)CT * D, rstd_c + (size_t)(t - 1) * CT);
            if constexpr (TOKEN) lgreg = TokenDecay<T, CT>::fetch(lg + (size_t)(t - 1) * CT);
        }
        // masked score tiles: dS^T = V dO^T (tiles 0..2) and S^T = K Q^T (tiles 3..5), one per wave
        {
            constexpr int NTRI = 3;  // lower-triangular 32x32 blocks of a 64x64 tile
#pragma unroll
            for (int idx = 0; idx < 2 * NTRI; ++idx) {
                if (idx % (2 * NW) != w8) continue;
                const int tri = idx % NTRI, ib = tri == 0 ? 0 : 1, jb = tri == 2 ? 1 : 0;
                const T *sA = idx < NTRI ? sV : sK, *sB = idx < NTRI ? sdO : sQ;
                f32x16 acc = {0}, acc2 = {0};
                pipelined<NKD / 2>(
                    [&](int s2) {
                        FragPair<FragPair<F>> f;
                        f.a.a = E::ld_kc(ln, sA, LDD, 32 * jb, 2 * s2 * E::KSTEP);
                        f.a.b = E::ld_kc(ln, sB, LDD, 32 * ib, 2 * s2 * E::KSTEP);
                        f.b.a = E::ld_kc(ln, sA, LDD, 32 * jb, (2 * s2 + 1) * E::KSTEP);
                        f.b.b = E::ld_kc(ln, sB, LDD, 32 * ib, (2 * s2 + 1) * E::KSTEP);
                        return f;
                    },
                    [&](int, const FragPair<FragPair<F>> &f) {
                        acc = E::mfma(f.a.a, f.a.b, acc);
                        acc2 = E::mfma(f.b.a, f.b.b, acc2);
                    });
                acc += acc2;
                store_masked_scores<T, LDP>(ln, idx < NTRI ? sDS : sS, acc, jb, ib, dec);
            }
        }
        __syncthreads();
        ln = fresh_lane();

        float rq = 0.0f;  // per-token decay: q_i . dq_i over this wave's features, tokens i of block 1 - rg
        // ---- dQ^T[a in w][i], tokens i of block 1 - rg:
        //      lambda^i sum_c KV_{t-1}[a][c] dO[i][c] + sum_{j<=i} K[j][a] dSm[i][j] ----
        {
            const int r0 = 32 * (1 - rg);   // group 0 takes the second token block (whose keys span both blocks), group 1 the first
            f32x16 acc = {0};
            pipelined<NKD>(
                [&](int ks) { return FragPair<F>{E::ld_kc(ln, sC, LDD, 32 * w, ks * E::KSTEP), E::ld_kc(ln, sdO, LDD, r0, ks * E::KSTEP)}; },
                [&](int, const FragPair<F> &f) { acc = E::mfma(f.a, f.b, acc); });
            acc *= dec.upto(r0 + ln.r);
            auto intra = [&](int ks) { return FragPair<F>{E::ld_ks(ln, sK, LDD, ks * E::KSTEP, 32 * w), E::ld_kc(ln, sDS, LDP, r0, ks * E::KSTEP)}; };
            auto fma = [&](int, const FragPair<F> &f) { acc = E::mfma(f.a, f.b, acc); };
            if (rg == 0) pipelined<2 * SPB>(intra, fma);    // keys of blocks 0 and 1
            else pipelined<SPB>(intra, fma);                // keys of block 0
            store_out_tile_t<T, D>(ln, dQ + off, acc, r0, w, nrows);
            if constexpr (TOKEN) rq = rowdot<T>(ln, acc, sQ, LDD, r0, w);
        }
        ln = fresh_lane();
        // ---- this group's product, both token blocks j (written for dV; dK is the same under K<->V, Q<->dO, S<->dS):
        //      dV^T[c in w][j] = lambda^(CT-j) sum_a dKV[a][c] K[j][a] + sum_{i>=j} dO[i][c] Sm[i][j] ----
        {
            f32x16 acc[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) acc[jb] = f32x16{0};
            struct Two { F b[NB]; };
            pipelined<DB * E::NSUB>(
                [&](int s2) {
                    Two f;
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb) f.b[jb] = E::ld_kp(ln, sX1, LDD, 32 * jb, 32 * (s2 / E::NSUB), s2 % E::NSUB);
                    return f;
                },
                [&](int s2, const Two &f) {
                    const F sf = E::from_acc(st[s2 / E::NSUB], s2 % E::NSUB);
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb) acc[jb] = E::mfma(sf, f.b[jb], acc[jb]);
                });
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) acc[jb] *= dec.after(32 * jb + ln.r);
            struct Three { F a; F b[NB]; };
            pipelined<NKS>(
                [&](int ks) {
                    Three f;
                    f.a = E::ld_ks(ln, sX2, LDD, ks * E::KSTEP, 32 * w);
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb)
                        if (jb <= ks / SPB) f.b[jb] = E::ld_ks(ln, sPm, LDP, ks * E::KSTEP, 32 * jb);
                    return f;
                },
                [&](int ks, const Three &f) {
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb)
                        if (jb <= ks / SPB) acc[jb] = E::mfma(f.a, f.b[jb], acc[jb]);
                });
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) store_out_tile_t<T, D>(ln, gOut + off, acc[jb], 32 * jb, w, nrows);
            if constexpr (TOKEN) {
#pragma unroll
                for (int jb = 0; jb < NB; ++jb) {
                    float r = jb == 1 - rg ? rq : 0.0f;
                    if (rg == 1) r -= rowdot<T>(ln, acc[jb], sK, LDD, 32 * jb, w);  // group 1 holds dK
                    if (ln.h == 0) rs[w8 * CT + 32 * jb + ln.r] = r;
                }
            }
        }
        ln = fresh_lane();
        // ---- state update in this group's orientation (group 0: dKV <- lambda^CT dKV + (Lambda Q)^T dO) ----
        {
            const float lamC = dec.whole();
#pragma unroll
            for (int blk = 0; blk < DB; ++blk) st[blk] *= lamC;
            struct Step {
                F b;
                F a[DB];
            };
            pipelined<NKS>(
                [&](int ks) {
                    Step f;
                    f.b = E::ld_ks(ln, sX2, LDD, ks * E::KSTEP, 32 * w);
#pragma unroll
                    for (int blk = 0; blk < DB; ++blk) f.a[blk] = E::ld_ks(ln, sUA, LDD, ks * E::KSTEP, 32 * blk);
                    return f;
                },
                [&](int ks, const Step &f) {
                    const F bs = dec.weigh_upto(ln, f.b, ks);
#pragma unroll
                    for (int blk = 0; blk < DB; ++blk) st[blk] = E::mfma(f.a[blk], bs, st[blk]);
                });
        }
    }
    if constexpr (TOKEN) {
        __syncthreads();
        flush_r(t0);
    }
    if (seg == 0 && rg == 0) state_store_w<D>(ln, st, dkv_in + (size_t)chain * D * D, w);
}

// ---------------------------------------------------------------------------
// k_bwd8p: k_bwd8 for a state cache that holds one state per PAIR of tiles
// (half the cache traffic of both passes). Tiles are walked in reverse as pairs
// (E = even tile, O = the odd tile after it). The cache gives KV at the start
// of E. The O tile's dQ needs the state one tile later,
//     KV_mid = lambda^CT KV + (diag{lambda^(CT-1-j)} K_E)^T V_E   (state update of Sec. 3.2);
// instead of rebuilding it, dQ of the O tile treats the pair as one chunk of 2 CT
// tokens (Alg. 3 with C = 2 CT, restricted to the rows of the O tile):
//     dQ_O = Lambda' dO_O KV^T + [(dO_O V_E^T) (.) M'] K_E + [(dO_O V_O^T) (.) M] K_O,
// Lambda'_i = lambda^(CT+i), M'_ij = lambda^(CT+i-j): one more masked score tile
// (sDX) and four more contraction steps, and the cached tile stays in LDS for
// both tiles. K_E, V_E are needed for the E tile anyway and are simply fetched
// one tile early. Per pair: six barriers, 9 tile loads, one cache-tile load.
// ---------------------------------------------------------------------------
template <typename T, int CT, int D>
struct Bwd8pSmem {
    static constexpr int LDD = tile_ld<T, D>(), LDP = CT + Elem<T>::PAD;
    static constexpr size_t TILE = (size_t)CT * LDD * sizeof(T);
    static constexpr size_t P_OFF = 6 * TILE;
    static constexpr size_t C_OFF = P_OFF + 3 * (size_t)CT * LDP * sizeof(T);   // S, dS and the cross tile dS(O x E)
    static constexpr size_t PW_OFF = C_OFF + (size_t)D * LDD * sizeof(T);
    // decay tables of the O tile and of the E tile, then one row of per-token partial sums per wave
    static constexpr size_t TOTAL = PW_OFF + (6 * CT + 4 + 8 * CT) * sizeof(float);
};

// WK, WV: elements per row of Q, K, dQ, dK and of V, dO, dV in memory (<= D; see k_local).
template <typename T, int CT, int D, bool TOKEN, bool NORM = false, int WK = D, int WV = D>
__global__ __launch_bounds__(D * 4) void k_bwd8p(const T *__restrict__ Q, const T *__restrict__ K,
                                                  const T *__restrict__ V, const T *__restrict__ dO,
                                                  const float *__restrict__ decay, const T *__restrict__ cache,
                                                  T *__restrict__ dQ, T *__restrict__ dK, T *__restrict__ dV,
                                                  float *__restrict__ dkv_in, const float *__restrict__ scratch,
                                                  float *__restrict__ rtok,
                                                  int H, int ntiles, int nseg, int tiles_per_seg, int ntok, int kvdiv,
                                                  const T *__restrict__ yn = nullptr, const float *__restrict__ rstd = nullptr) {
    using E = Elem<T>;
    using F = typename E::frag;
    using SM = Bwd8pSmem<T, CT, D>;
    static_assert(CT == 64, "two 32-token blocks per tile");
    constexpr int NT = D * 4, NW = D / 32, LDD = SM::LDD, LDP = SM::LDP, DB = D / 32, NB = CT / 32, NKS = CT / E::KSTEP,
                  NKD = D / E::KSTEP, SPB = 32 / E::KSTEP;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    T *sVO = (T *)smem;            // V of the O tile
    T *sdO = sVO + CT * LDD;       // dO of the tile being processed
    T *sKO = sdO + CT * LDD;       // K of the O tile
    T *sQ = sKO + CT * LDD;        // Q of the tile being processed
    T *sVE = sQ + CT * LDD;        // V of the E tile
    T *sKE = sVE + CT * LDD;       // K of the E tile
    T *sS = (T *)(smem + SM::P_OFF);
    T *sDS = sS + CT * LDP;
    T *sDX = sDS + CT * LDP;       // masked dS between the O tile's queries and the E tile's keys
    T *sC = (T *)(smem + SM::C_OFF);
    float *pw = (float *)(smem + SM::PW_OFF);

    const int chain = blockIdx.y, seg = blockIdx.x;
    const int t0 = seg * tiles_per_seg;                 // even
    const int t1 = min(t0 + tiles_per_seg, ntiles);     // even
    const int w8 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int w = w8 % NW;    // feature block of this wave's outputs
    const int rg = w8 / NW;   // group: 0 produces dV, 1 produces dK
    Lane ln = fresh_lane();

    K += kv_shift(chain, H, kvdiv, ntok, WK);   // K, V of this chain's K/V head
    V += kv_shift(chain, H, kvdiv, ntok, WV);
    auto koff = [&](int t) { return tile_off(chain, ntok, t, CT, WK); };
    auto voff = [&](int t) { return tile_off(chain, ntok, t, CT, WV); };
    TileMover<T, CT, D, NT> mvO, moX, mkO, mqX, mvE, mkE;   // moX / mqX carry dO, Q of the O tile, then of the E tile
    TileMover<T, D, D, NT> mc;                               // cached state at the start of the E tile
    const T *ctile = cache + (size_t)chain * (ntiles / 2) * WK * WV;   // [WK][WV] per slot
    // With a decay per token (`decay` = log g, [chain][token]) the O and the E tile have their own
    // tables; with one lambda per head both names refer to the same table.
    const auto decO = DecaySel<TOKEN, T, CT>::make(pw, decay, chain, H);
    const auto decE = [&] {
        if constexpr (TOKEN) return TokenDecay<T, CT>(pw + 3 * CT);
        else return decO;
    }();
    // weight key j of the E tile carries at query i of the O tile, and the E tile's entering state at query i
    // (one lambda per head: powers CT+1 .. 2 CT of the same table)
    auto cross_weight = [&](int i, int j) {
        if constexpr (TOKEN) return decO.upto(i) * decE.after(j);
        else return decO.pw[CT + i - j];
    };
    auto far_upto = [&](int i) {
        if constexpr (TOKEN) return decO.upto(i) * decE.whole();
        else return decO.pw[CT + i + 1];
    };
    const float *lg = decay + (size_t)chain * ntok;
    typename TokenDecay<T, CT>::LogG lgO = {}, lgE = {};
    // per-token decay: r_t = q_t.dq_t - k_t.dk_t, one partial row per wave, summed and written per tile
    float *rs = pw + 6 * CT + 4;
    auto flush_r = [&](int tile) {
        if (threadIdx.x < CT) {
            float r = 0.0f;
#pragma unroll
            for (int wv = 0; wv < 2 * NW; ++wv) r += rs[wv * CT + threadIdx.x];
            if (tile * CT + (int)threadIdx.x < ntok) rtok[(size_t)chain * ntok + (size_t)tile * CT + threadIdx.x] = r;
        }
    };
    NormTile<T, CT, D, NT, WV> mnX;  // NORM: partner of moX (dO is dY; see NormTile)
    const float *rstd_c = rstd + (size_t)chain * ntok;
    // The requests for a pair come in two parts. K and V of both tiles go into registers that are idle
    // from the top of an iteration on, so inside the loop they are issued a whole tile early (during
    // the O tile of the pair before); dO, Q of the O tile and the cached state follow once the E tile
    // of the pair before has taken their registers' contents. Fewer requests are then issued in one
    // burst, which is where the waves stall at the memory pipeline's entry.
    auto load_pair_kv = [&](int tE) {
        const int nvO = TOKEN ? min(CT, ntok - (tE + 1) * CT) : CT;   // only the O tile of the last pair can be short
        mvO.template load_w<WV>(V + voff(tE + 1), nvO);
        mkO.template load_w<WK>(K + koff(tE + 1), nvO);
        mvE.template load_w<WV>(V + voff(tE), CT);
        mkE.template load_w<WK>(K + koff(tE), CT);
        mc.template load_w<WV>(ctile + (size_t)(tE / 2) * WK * WV, WK);   // rows and columns of padding read as zero
    };
    auto load_pair_rest = [&](int tE) {
        const int nvO = TOKEN ? min(CT, ntok - (tE + 1) * CT) : CT;
        if constexpr (NORM) mnX.load(yn + voff(tE + 1), rstd_c + (size_t)(tE + 1) * CT, nvO);
        if constexpr (TOKEN) {
            lgO = TokenDecay<T, CT>::fetch(lg + (size_t)(tE + 1) * CT, nvO);
            lgE = TokenDecay<T, CT>::fetch(lg + (size_t)tE * CT);
        }
        moX.template load_w<WV>(dO + voff(tE + 1), nvO);
        mqX.template load_w<WK>(Q + koff(tE + 1), nvO);
    };
    auto load_pair = [&](int tE) {
        load_pair_kv(tE);
        load_pair_rest(tE);
    };
    load_pair(t1 - 2);

    const T *sX2 = rg ? sQ : sdO;    // intra operand and state-update B operand: [token][feature in w]
    const T *sUA = rg ? sdO : sQ;    // state-update A operand: [token][feature of the state rows]
    const T *sPm = rg ? sDS : sS;    // masked score tile of this group's product
    T *gOut = rg ? dK : dV;

    // st[blk][i]: group 0: dKV[32 blk + acc_row(i)][32 w + r]; group 1: dKV[32 w + r][32 blk + acc_row(i)]
    f32x16 st[DB];
    {
        const float *g = scratch + ((size_t)chain * nseg + seg) * WK * WV;
        if (rg == 0) state_load_w<D, WK, WV>(ln, st, g, w);
        else state_load_t_w<D, WK, WV>(ln, st, g, w);
    }

    // masked score tiles of the tile whose V, K are at pV, pK (dO, Q in sdO, sQ): one 32x32 block per wave
    // The O tile's queries against the E tile's keys: dSX^T[j][i] = sum_c V_E[j][c] dO_O[i][c], all four
    // 32x32 blocks, weighted and stored as sDX[i][j]. Two blocks go to the two waves that have no
    // triangular block, one each to two waves of group 0.
    auto cross_scores = [&]() {
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
            const int owner = blk < 2 ? 6 + blk : blk;   // waves 6, 7, 2, 3
            if (owner % (2 * NW) != w8) continue;
            const int ib = blk >> 1, jb = blk & 1;
            f32x16 acc = {0}, acc2 = {0};
            pipelined<WV / E::KSTEP / 2>(   // (contraction over the real value features)
                [&](int s2) {
                    FragPair<FragPair<F>> f;
                    f.a.a = E::ld_kc(ln, sVE, LDD, 32 * jb, 2 * s2 * E::KSTEP);
                    f.a.b = E::ld_kc(ln, sdO, LDD, 32 * ib, 2 * s2 * E::KSTEP);
                    f.b.a = E::ld_kc(ln, sVE, LDD, 32 * jb, (2 * s2 + 1) * E::KSTEP);
                    f.b.b = E::ld_kc(ln, sdO, LDD, 32 * ib, (2 * s2 + 1) * E::KSTEP);
                    return f;
                },
                [&](int, const FragPair<FragPair<F>> &f) {
                    acc = E::mfma(f.a.a, f.a.b, acc);
                    acc2 = E::mfma(f.b.a, f.b.b, acc2);
                });
            acc += acc2;
            const int iq = 32 * ib + ln.r;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int j0 = 32 * jb + 8 * g + 4 * ln.h;
                float x[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = acc[4 * g + e] * cross_weight(iq, j0 + e);
                E::st4(sDX + iq * LDP + j0, x[0], x[1], x[2], x[3]);
            }
        }
    };
    auto scores = [&](const auto &dec, const T *pV, const T *pK) {
        constexpr int NTRI = 3;
#pragma unroll
        for (int idx = 0; idx < 2 * NTRI; ++idx) {
            if (idx % (2 * NW) != w8) continue;
            const int tri = idx % NTRI, ib = tri == 0 ? 0 : 1, jb = tri == 2 ? 1 : 0;
            const T *sA = idx < NTRI ? pV : pK, *sB = idx < NTRI ? sdO : sQ;
            f32x16 acc = {0}, acc2 = {0};
            auto contract = [&](auto steps) __attribute__((always_inline)) {
                pipelined<decltype(steps)::value>(
                    [&](int s2) {
                        FragPair<FragPair<F>> f;
                        f.a.a = E::ld_kc(ln, sA, LDD, 32 * jb, 2 * s2 * E::KSTEP);
                        f.a.b = E::ld_kc(ln, sB, LDD, 32 * ib, 2 * s2 * E::KSTEP);
                        f.b.a = E::ld_kc(ln, sA, LDD, 32 * jb, (2 * s2 + 1) * E::KSTEP);
                        f.b.b = E::ld_kc(ln, sB, LDD, 32 * ib, (2 * s2 + 1) * E::KSTEP);
                        return f;
                    },
                    [&](int, const FragPair<FragPair<F>> &f) {
                        acc = E::mfma(f.a.a, f.a.b, acc);
                        acc2 = E::mfma(f.b.a, f.b.b, acc2);
                    });
            };
            // dS = dO V^T contracts over the real value features, S = Q K^T over the real key features
            if (idx < NTRI) contract(std::integral_constant<int, WV / E::KSTEP / 2>{});
            else contract(std::integral_constant<int, WK / E::KSTEP / 2>{});
            acc += acc2;
            store_masked_scores<T, LDP>(ln, idx < NTRI ? sDS : sS, acc, jb, ib, dec);
        }
    };

    // dQ, this group's dV or dK, and the dKV update for tile `t`
    // `cross` (the O tile): the cached state is the one the E tile starts from, so dQ takes the E tile
    // as the first half of its own chunk: far weights on the state term, plus the E tile's keys through sDX.
    // Key and value dimensions that differ: only KB (VB) of the DB 32-wide feature blocks of the key (value)
    // side are real. A wave whose own output block (dV block w in group 0, dK block w in group 1) is padding
    // skips that product and its state update. With d_k < d_v the two such waves of group 1 produce ALL of
    // dQ instead (both token blocks of one key-feature block each), so that no wave carries dQ on top of a
    // dK or dV block and a state update (the walk's critical path); otherwise every wave with a real
    // key-feature block produces the dQ tile of that block for one token block (group 0 the second, whose
    // keys span both blocks, group 1 the first).
    constexpr int KB = WK / 32, VB = WV / 32;
    const bool own_block = WK == WV || (rg ? w < KB : w < VB);   // this wave's dK / dV block exists
    constexpr bool DQ_BY_IDLE = WK < WV && !(TOKEN && NORM);   // (that one combination would run out of registers)
    auto products = [&](const auto &dec, const T *pV, const T *pK, int t, int nrows, bool cross) {
        const T *sX1 = rg ? pV : pK;  // inter operand: token rows, features contracted with the state
        float rq[NB] = {};  // per-token decay: q_i . dq_i over the features of the dQ tiles this wave produced, per token block
        // dQ^T[a in block qa][i], tokens i of the block starting at r0; `both`: the intra part reaches the keys of
        // both blocks (the second token block) or of block 0 only
        auto dq_tile = [&](int qa, int r0, auto both) __attribute__((always_inline)) {
            f32x16 acc = {0};
            pipelined<WV / E::KSTEP>(   // (the cached state's real columns)
                [&](int ks) { return FragPair<F>{E::ld_kc(ln, sC, LDD, 32 * qa, ks * E::KSTEP), E::ld_kc(ln, sdO, LDD, r0, ks * E::KSTEP)}; },
                [&](int, const FragPair<F> &f) { acc = E::mfma(f.a, f.b, acc); });
            acc *= cross ? far_upto(r0 + ln.r) : dec.upto(r0 + ln.r);
            auto fma = [&](int, const FragPair<F> &f) { acc = E::mfma(f.a, f.b, acc); };
            if (cross)
                pipelined<NKS>(
                    [&](int ks) { return FragPair<F>{E::ld_ks(ln, sKE, LDD, ks * E::KSTEP, 32 * qa), E::ld_kc(ln, sDX, LDP, r0, ks * E::KSTEP)}; },
                    fma);
            auto intra = [&](int ks) { return FragPair<F>{E::ld_ks(ln, pK, LDD, ks * E::KSTEP, 32 * qa), E::ld_kc(ln, sDS, LDP, r0, ks * E::KSTEP)}; };
            pipelined<decltype(both)::value ? 2 * SPB : SPB>(intra, fma);
            if constexpr (TOKEN) rq[r0 / 32] = rowdot<T>(ln, acc, sQ, LDD, r0, qa);   // (from the fp32 accumulators, before rounding)
            store_out_tile_t<T, D, WK>(ln, dQ + koff(t), acc, r0, qa, nrows);
        };
        if constexpr (DQ_BY_IDLE) {
            if (rg == 1 && w >= KB) {
                dq_tile(w - KB, 32, std::true_type{});
                dq_tile(w - KB, 0, std::false_type{});
            }
        } else if (WK == WV || w < KB) {
            if (rg == 0) dq_tile(w, 32, std::true_type{});
            else dq_tile(w, 0, std::false_type{});
        }
        ln = fresh_lane();
        if (own_block) {   // dV^T[c in w][j] (group 0) or dK^T[a in w][j] (group 1), both token blocks
            f32x16 acc[NB];
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) acc[jb] = f32x16{0};
            struct Two { F b[NB]; };
            pipelined<DB * E::NSUB>(
                [&](int s2) {
                    Two f;
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb) f.b[jb] = E::ld_kp(ln, sX1, LDD, 32 * jb, 32 * (s2 / E::NSUB), s2 % E::NSUB);
                    return f;
                },
                [&](int s2, const Two &f) {
                    const F sf = E::from_acc(st[s2 / E::NSUB], s2 % E::NSUB);
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb) acc[jb] = E::mfma(sf, f.b[jb], acc[jb]);
                });
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) acc[jb] *= dec.after(32 * jb + ln.r);
            struct Three { F a; F b[NB]; };
            pipelined<NKS>(
                [&](int ks) {
                    Three f;
                    f.a = E::ld_ks(ln, sX2, LDD, ks * E::KSTEP, 32 * w);
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb)
                        if (jb <= ks / SPB) f.b[jb] = E::ld_ks(ln, sPm, LDP, ks * E::KSTEP, 32 * jb);
                    return f;
                },
                [&](int ks, const Three &f) {
#pragma unroll
                    for (int jb = 0; jb < NB; ++jb)
                        if (jb <= ks / SPB) acc[jb] = E::mfma(f.a, f.b[jb], acc[jb]);
                });
#pragma unroll
            for (int jb = 0; jb < NB; ++jb) {
                if constexpr (TOKEN) {   // (row dots from the fp32 accumulators, before they are rounded and stored)
                    float r = rq[jb];
                    if (rg == 1) r -= rowdot<T>(ln, acc[jb], pK, LDD, 32 * jb, w);  // group 1 holds dK
                    if (ln.h == 0) rs[w8 * CT + 32 * jb + ln.r] = r;
                }
                if constexpr (WK == WV) {
                    store_out_tile_t<T, D, WK>(ln, gOut + koff(t), acc[jb], 32 * jb, w, nrows);
                } else {
                    if (rg) store_out_tile_t<T, D, WK>(ln, dK + koff(t), acc[jb], 32 * jb, w, nrows);
                    else store_out_tile_t<T, D, WV>(ln, dV + voff(t), acc[jb], 32 * jb, w, nrows);
                }
            }
        } else if constexpr (TOKEN) {   // this wave's row of the per-token sums still has to be defined
#pragma unroll
            for (int jb = 0; jb < NB; ++jb)
                if (ln.h == 0) rs[w8 * CT + 32 * jb + ln.r] = rq[jb];
        }
        ln = fresh_lane();
        if (own_block) {   // state update in this group's orientation
            const float lamC = dec.whole();
#pragma unroll
            for (int blk = 0; blk < DB; ++blk) st[blk] *= lamC;
            struct Step { F b; F a[DB]; };
            pipelined<NKS>(
                [&](int ks) {
                    Step f;
                    f.b = E::ld_ks(ln, sX2, LDD, ks * E::KSTEP, 32 * w);
#pragma unroll
                    for (int blk = 0; blk < DB; ++blk) f.a[blk] = E::ld_ks(ln, sUA, LDD, ks * E::KSTEP, 32 * blk);
                    return f;
                },
                [&](int ks, const Step &f) {
                    const F bs = dec.weigh_upto(ln, f.b, ks);
#pragma unroll
                    for (int blk = 0; blk < DB; ++blk) st[blk] = E::mfma(f.a[blk], bs, st[blk]);
                });
        }
    };

    for (int tE = t1 - 2; tE >= t0; tE -= 2) {
        __syncthreads();  // previous pair fully consumed
        ln = fresh_lane();
        if constexpr (TOKEN) {
            if (tE + 2 < t1) flush_r(tE + 2);  // E tile of the previous pair
            decO.fill(lgO);
            decE.fill(lgE);
        }
        if constexpr (NORM) mnX.apply(moX);
        mvO.store(sVO, LDD);
        moX.store(sdO, LDD);
        mkO.store(sKO, LDD);
        mqX.store(sQ, LDD);
        mvE.store(sVE, LDD);
        mkE.store(sKE, LDD);
        mc.store(sC, LDD);   // the state the E tile starts from serves both tiles of the pair
        if (tE > t0) load_pair_kv(tE - 2);
        __syncthreads();
        ln = fresh_lane();
        moX.template load_w<WV>(dO + voff(tE), CT);
        mqX.template load_w<WK>(Q + koff(tE), CT);
        if constexpr (NORM) mnX.load(yn + voff(tE), rstd_c + (size_t)tE * CT);
        // ---- O tile ----
        scores(decO, sVO, sKO);
        cross_scores();
        __syncthreads();
        ln = fresh_lane();
        products(decO, sVO, sKO, tE + 1, TOKEN ? min(CT, ntok - (tE + 1) * CT) : CT, true);
        __syncthreads();  // O tile consumed: sdO, sQ are free
        ln = fresh_lane();
        if constexpr (TOKEN) flush_r(tE + 1);
        if constexpr (NORM) mnX.apply(moX);
        moX.store(sdO, LDD);
        mqX.store(sQ, LDD);
        __syncthreads();
        ln = fresh_lane();
        if (tE > t0) load_pair_rest(tE - 2);
        // ---- E tile ----
        scores(decE, sVE, sKE);
        __syncthreads();
        ln = fresh_lane();
        products(decE, sVE, sKE, tE, CT, false);
    }
    if constexpr (TOKEN) {
        __syncthreads();
        flush_r(t0);
    }
    if (seg == 0 && rg == 0) state_store_w<D, WK, WV>(ln, st, dkv_in + (size_t)chain * WK * WV, w);
}

// ---------------------------------------------------------------------------
// k_dlg: gradient of the per-token log decay from r_t = q_t.dq_t - k_t.dk_t
// (written per tile by the backward walk):
//     dlog g_s = <dkv_out, kv_out> + sum_{t >= s} r_t.
// It follows from expanding <D_s, kv_s> with either recurrence, kv_s = g_s kv_{s-1}
// + k_s v_s^T or D_s = q_s do_s^T + g_{s+1} D_{s+1} (D_s: gradient w.r.t. kv_s):
// dlog g_s + k_s.dk_s = q_s.dq_s + dlog g_{s+1}. One workgroup per block of
// kDlgBlock tokens of a head: it sums everything behind its block (r of the later
// tokens and the boundary term), then scans its own tokens from the right. Sums
// are carried in double; the order of additions is fixed, so reruns are identical.
// ---------------------------------------------------------------------------
constexpr int kDlgBlock = 1024;  // tokens per workgroup: 256 threads x 4

DEVI double block_sum(double x, double *sh) {  // sum over the 256 threads, returned to all
    const int tid = threadIdx.x;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    __syncthreads();
    if ((tid & 63) == 0) sh[tid >> 6] = x;
    __syncthreads();
    return sh[0] + sh[1] + sh[2] + sh[3];
}

__global__ __launch_bounds__(256) void k_dlg(const float *__restrict__ rtok, const float *__restrict__ kv_out,
                                             const float *__restrict__ dkv_out, float *__restrict__ dlg, int N, int DD) {
    __shared__ double sh[4];
    const int chain = blockIdx.y, tid = threadIdx.x;
    const int s0 = blockIdx.x * kDlgBlock;  // first token of this block
    const float *r = rtok + (size_t)chain * N;
    double behind = 0.0;
    if (dkv_out) {
        const f32x4 *a = (const f32x4 *)(kv_out + (size_t)chain * DD), *b = (const f32x4 *)(dkv_out + (size_t)chain * DD);
        for (int e = tid; e < DD / 4; e += 256) {
            const f32x4 x = a[e], y = b[e];
            behind += (double)x[0] * y[0] + (double)x[1] * y[1] + (double)x[2] * y[2] + (double)x[3] * y[3];
        }
    }
    if (N % 4 == 0) {   // rows of r are 16-byte aligned: four tokens per load, four loads in flight
        double b1 = 0.0, b2 = 0.0, b3 = 0.0;
        int s = s0 + kDlgBlock + 4 * tid;
        for (; s + 3 * kDlgBlock < N; s += 4 * kDlgBlock) {
            const f32x4 x0 = *(const f32x4 *)(r + s), x1 = *(const f32x4 *)(r + s + kDlgBlock),
                        x2 = *(const f32x4 *)(r + s + 2 * kDlgBlock), x3 = *(const f32x4 *)(r + s + 3 * kDlgBlock);
            behind += ((double)x0[0] + x0[1]) + ((double)x0[2] + x0[3]);
            b1 += ((double)x1[0] + x1[1]) + ((double)x1[2] + x1[3]);
            b2 += ((double)x2[0] + x2[1]) + ((double)x2[2] + x2[3]);
            b3 += ((double)x3[0] + x3[1]) + ((double)x3[2] + x3[3]);
        }
        for (; s < N; s += kDlgBlock) {
            const f32x4 x = *(const f32x4 *)(r + s);
            behind += ((double)x[0] + x[1]) + ((double)x[2] + x[3]);
        }
        behind += (b1 + b2) + b3;
    } else {
        for (int s = s0 + kDlgBlock + tid; s < N; s += 256) behind += (double)r[s];
    }
    behind = block_sum(behind, sh);
    // this thread's four tokens, suffix sums inside the group
    const int s = s0 + 4 * tid;
    float x[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = s + e < N ? r[s + e] : 0.0f;
    double v3 = x[3], v2 = v3 + x[2], v1 = v2 + x[1], v0 = v1 + x[0];
    // exclusive suffix sum of the group totals over the threads behind this one
    double incl = v0;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const double y = __shfl_down(incl, d, 64);
        if ((tid & 63) + d < 64) incl += y;
    }
    __syncthreads();
    if ((tid & 63) == 0) sh[tid >> 6] = incl;  // total of this wave
    __syncthreads();
    double after = behind + (incl - v0);
    for (int wv = (tid >> 6) + 1; wv < 4; ++wv) after += sh[wv];
    const double v[4] = {v0, v1, v2, v3};
    float *o = dlg + (size_t)chain * N;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (s + e < N) o[s + e] = (float)(after + v[e]);
}

// ---------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------
template <typename T, int CT, int D>
struct Smem {
    using E = Elem<T>;
    static constexpr size_t local = 2 * (size_t)CT * tile_ld<T, D>() * sizeof(T) + table_floats<CT>() * sizeof(float);
    static constexpr size_t fwd = (3 * (size_t)CT * tile_ld<T, D>() + (size_t)CT * (CT + E::PAD)) * sizeof(T) + table_floats<CT>() * sizeof(float);
    static constexpr size_t bwd = BwdSmem<T, CT, D>::TOTAL;
    static_assert(fwd <= 163840 && bwd <= 163840, "LDS budget of one gfx950 CU exceeded");
};

// One launch of a kernel with `lds` bytes of dynamic LDS. Kernels that need more than the 64 KB default
// have their limit raised first (once per kernel and device, see allow_dynamic_lds).
template <typename... KArgs, typename... Args>
static hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t s, Args... args) {
    if (hipError_t e = allow_dynamic_lds((const void *)kernel, lds); e != hipSuccess) return e;
    kernel<<<grid, block, lds, s>>>(args...);
    return hipSuccess;
}

// A kernel family instantiated for both decay models, with and without the fused Norm: picks the
// member that serves the plan. Fam::fn<TOKEN, NORM> is the kernel.
template <typename Fam>
static auto by_model(const Plan &p) {
    return p.token ? (p.norm ? Fam::template fn<true, true> : Fam::template fn<true, false>)
                   : (p.norm ? Fam::template fn<false, true> : Fam::template fn<false, false>);
}

// Grouped K/V heads, backward: the walking kernel wrote dK, dV per QUERY head into `part`
// ([chains][ntok][D], in the data type, so each partial gradient is already rounded to it once);
// dK, dV of a K/V head are the sums over its kvdiv query heads, added in fp32 in a fixed order and
// rounded to the data type a second time. For bfloat16 the partials' rounding errors (2^-9 relative
// each, independent) add in quadrature, so the sum stays well inside the 2e-2 bound also for
// multi-query attention (tested with 16 query heads per K/V head).
template <typename T>
__global__ __launch_bounds__(256) void k_group_sum(const T *__restrict__ part, T *__restrict__ out, int kvdiv, size_t per_head) {
    const size_t kvchain = blockIdx.y;
    const T *src = part + kvchain * kvdiv * per_head;
    T *dst = out + kvchain * per_head;
    for (size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4; e < per_head; e += (size_t)gridDim.x * 256 * 4) {
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int g = 0; g < kvdiv; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] += Elem<T>::ld1(src + (size_t)g * per_head + e + i);
        Elem<T>::st4(dst + e, acc[0], acc[1], acc[2], acc[3]);   // per_head = ntok * D is a multiple of 4
    }
}
template <typename T>
static hipError_t run_group_sum(const Plan &p, const void *part, void *out, int width, hipStream_t s) {
    const size_t per_head = (size_t)p.N * width;
    const int kvchains = p.B * (p.H / p.kvdiv);
    size_t blocks = (per_head / 4 + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    k_group_sum<T><<<dim3((unsigned)blocks, kvchains), dim3(256), 0, s>>>((const T *)part, (T *)out, p.kvdiv, per_head);
    return hipGetLastError();
}

// Kernel families by decay model and Norm (see by_model).
template <typename T, int CT, int D, bool BWD, bool WITH_NORM, int WX, int WY>
struct LocalFam {   // the Norm prologue exists in the backward pass only
    template <bool TK, bool NM>
    static constexpr auto fn = k_local<T, CT, D, BWD, TK, NM && BWD && WITH_NORM, WX, WY>;
};
template <typename T, int CT, int D, int WK, int WV>
struct FwdFam {
    template <bool TK, bool NM>
    static constexpr auto fn = k_fwd<T, CT, D, TK, NM, WK, WV>;
};
template <typename T, int CT, int D, int WK, int WV>
struct StatesFam {  // the forward walk reduced to the states (no Norm: the states do not depend on it)
    template <bool TK, bool NM>
    static constexpr auto fn = k_fwd<T, CT, D, TK, false, WK, WV, true>;
};
template <typename T, int CT, int D, int WK, int WV>
struct BwdFam {     // four waves, one cached state per tile
    template <bool TK, bool NM>
    static constexpr auto fn = k_bwd<T, CT, D, TK, NM, WK, WV>;
};
template <typename T, int CT, int D>
struct Bwd8Fam {    // eight waves, one cached state per tile
    template <bool TK, bool NM>
    static constexpr auto fn = k_bwd8<T, CT, D, TK, NM>;
};
template <typename T, int CT, int D, int WK, int WV>
struct Bwd8pFam {   // eight waves, one cached state per pair of tiles
    template <bool TK, bool NM>
    static constexpr auto fn = k_bwd8p<T, CT, D, TK, NM, WK, WV>;
};

// The local pass only sums over its segment, so its tile need not be the walk's:
// bfloat16 segments made of an even number of 64-token tiles are read 128 tokens
// at a time (half the barriers, twice the bytes in flight per workgroup), unless
// the Norm prologue (a third tile in registers) or key and value dimensions that
// differ ask for the walk's tile.
template <typename T, int CT, int D, bool BWD, int WK = D, int WV = D>
static hipError_t run_local(const Plan &p, const T *x, const T *y, const float *decay, float *scratch, float *seglog,
                            const T *yn, const float *rstd, hipStream_t s) {
    const dim3 grid(p.nseg - 1, p.B * p.H), block(D * 2);
    if constexpr (sizeof(T) == 2 && CT == 64 && WK == D && WV == D) {
        if (!(BWD && p.norm) && p.tiles_per_seg % 2 == 0 && p.ntiles % 2 == 0)
            return launch_kernel(by_model<LocalFam<T, 128, D, BWD, false, D, D>>(p), grid, block, Smem<T, 128, D>::local, s, x, y,
                                 decay, scratch, seglog, p.H, p.ntiles / 2, p.nseg, p.tiles_per_seg / 2, p.N, p.kvdiv,
                                 (const T *)nullptr, (const float *)nullptr);
    }
    return launch_kernel(by_model<LocalFam<T, CT, D, BWD, true, WK, WV>>(p), grid, block, Smem<T, CT, D>::local, s, x, y, decay,
                         scratch, seglog, p.H, p.ntiles, p.nseg, p.tiles_per_seg, p.N, p.kvdiv, yn, rstd);
}

template <typename T, int CT, int D, int WK = D, int WV = D>
static hipError_t run_fwd(const Plan &p, const FwdArgs &a, hipStream_t s, const KernelEvents *ke) {
    const int chains = p.B * p.H, DD = WK * WV;   // states hold the real rows and columns only
    const dim3 scan_grid((DD / 4 + 255) / 256, chains);
    hipError_t e;
    if (ke) (void)hipEventRecord(ke->ev[0], s);
    if (p.nseg > 1) {
        if (e = run_local<T, CT, D, false, WK, WV>(p, (const T *)a.k, (const T *)a.v, a.decay, a.scratch, a.seglog, nullptr, nullptr, s);
            e != hipSuccess)
            return e;
    }
    if (ke) (void)hipEventRecord(ke->ev[1], s);
    if (p.token)
        k_scan<false, true><<<scan_grid, dim3(256), 0, s>>>(a.scratch, a.kv_in, nullptr, a.seglog, p.H, DD, p.nseg,
                                                           p.tiles_per_seg, p.ntiles, p.tile);
    else
        k_scan<false, false><<<scan_grid, dim3(256), 0, s>>>(a.scratch, a.kv_in, a.decay, nullptr, p.H, DD, p.nseg,
                                                            p.tiles_per_seg, p.ntiles, p.tile);
    if (ke) (void)hipEventRecord(ke->ev[2], s);
    const auto walk = a.states_only ? by_model<StatesFam<T, CT, D, WK, WV>>(p) : by_model<FwdFam<T, CT, D, WK, WV>>(p);
    if (e = launch_kernel(walk, dim3(p.nseg, chains), dim3(D * 2), Smem<T, CT, D>::fwd, s,
                          (const T *)a.q, (const T *)a.k, (const T *)a.v, a.decay, (T *)a.out, a.kv_out, (T *)a.cache,
                          (const float *)a.scratch, p.H, p.ntiles, p.nseg, p.tiles_per_seg, p.cache_stride, p.N, p.kvdiv,
                          a.rstd_out, a.eps);
        e != hipSuccess)
        return e;
    if (ke) (void)hipEventRecord(ke->ev[3], s);
    return hipGetLastError();
}

template <typename T, int CT, int D, int WK = D, int WV = D>
static hipError_t run_bwd(const Plan &p, const BwdArgs &a, hipStream_t s, const KernelEvents *ke) {
    const int chains = p.B * p.H, DD = WK * WV;   // states hold the real rows and columns only
    const dim3 scan_grid((DD / 4 + 255) / 256, chains);
    hipError_t e;
    if (ke) (void)hipEventRecord(ke->ev[0], s);
    if (p.nseg > 1) {
        if (e = run_local<T, CT, D, true, WK, WV>(p, (const T *)a.q, (const T *)a.dout, a.decay, a.scratch, a.seglog, (const T *)a.yn,
                                          a.rstd, s);
            e != hipSuccess)
            return e;
    }
    if (ke) (void)hipEventRecord(ke->ev[1], s);
    if (p.token)
        k_scan<true, true><<<scan_grid, dim3(256), 0, s>>>(a.scratch, a.dkv_out, nullptr, a.seglog, p.H, DD, p.nseg,
                                                          p.tiles_per_seg, p.ntiles, p.tile);
    else
        k_scan<true, false><<<scan_grid, dim3(256), 0, s>>>(a.scratch, a.dkv_out, a.decay, nullptr, p.H, DD, p.nseg,
                                                           p.tiles_per_seg, p.ntiles, p.tile);
    if (ke) (void)hipEventRecord(ke->ev[2], s);
    // The walking kernel: bfloat16 tiles of 64 tokens run in eight waves, with one cached state per pair of
    // tiles when the tile count is even; everything else in four waves with one cached state per tile. All
    // three take the same arguments. (Only the kernels a shape can reach are instantiated.)
    typedef void (*Walk)(const T *, const T *, const T *, const T *, const float *, const T *, T *, T *, T *, float *,
                         const float *, float *, int, int, int, int, int, int, const T *, const float *);
    Walk walk = nullptr;
    unsigned threads = D * 2;
    size_t lds = Smem<T, CT, D>::bwd;
    constexpr bool kEightWaves = sizeof(T) == 2 && CT == 64, kEqualDims = WK == D && WV == D;
    if constexpr (kEightWaves) {
        static_assert(Bwd8pSmem<T, CT, D>::TOTAL <= 163840 && Bwd8Smem<T, CT, D>::TOTAL <= 163840, "LDS budget of one gfx950 CU exceeded");
        if (p.cache_stride == 2) {
            walk = by_model<Bwd8pFam<T, CT, D, WK, WV>>(p);
            threads = D * 4;
            lds = Bwd8pSmem<T, CT, D>::TOTAL;
        } else if constexpr (kEqualDims) {
            walk = by_model<Bwd8Fam<T, CT, D>>(p);
            threads = D * 4;
            lds = Bwd8Smem<T, CT, D>::TOTAL;
        } else {
            walk = by_model<BwdFam<T, CT, D, WK, WV>>(p);
        }
    } else {
        walk = by_model<BwdFam<T, CT, D, WK, WV>>(p);
    }
    if (e = launch_kernel(walk, dim3(p.nseg, chains), dim3(threads), lds, s, (const T *)a.q, (const T *)a.k, (const T *)a.v,
                          (const T *)a.dout, a.decay, (const T *)a.cache, (T *)a.dq, (T *)a.dk, (T *)a.dv, a.dkv_in,
                          (const float *)a.scratch, a.rtok, p.H, p.ntiles, p.nseg, p.tiles_per_seg, p.N, p.kvdiv,
                          (const T *)a.yn, a.rstd);
        e != hipSuccess)
        return e;
    if (p.kvdiv > 1) {
        if (e = run_group_sum<T>(p, a.dk, a.dk_out, p.dk, s); e != hipSuccess) return e;
        if (e = run_group_sum<T>(p, a.dv, a.dv_out, p.dv, s); e != hipSuccess) return e;
    }
    if (ke) (void)hipEventRecord(ke->ev[3], s);
    if (p.token && a.dlog_g)
        k_dlg<<<dim3((p.N + kDlgBlock - 1) / kDlgBlock, chains), dim3(256), 0, s>>>(a.rtok, a.kv_out, a.dkv_out, a.dlog_g,
                                                                                      p.N, WK * WV);
    return hipGetLastError();
}

// log g = log(lambda_h) for every token of head h: lets a sub-sequence whose length is not a multiple of
// the tile run through the per-token-decay kernels (which handle a short last tile) with one lambda per head.
__global__ __launch_bounds__(256) void k_fill_logg(const float *__restrict__ decay, float *__restrict__ log_g, int H, int N) {
    const int chain = blockIdx.y;
    const float x = (float)log((double)decay[chain % H]);
    for (int s = blockIdx.x * 256 + threadIdx.x; s < N; s += gridDim.x * 256) log_g[(size_t)chain * N + s] = x;
}
hipError_t launch_fill_logg(const Plan &p, const float *decay, float *log_g, hipStream_t stream) {
    k_fill_logg<<<dim3((p.N + 255) / 256 < 64 ? (p.N + 255) / 256 : 64, p.B * p.H), dim3(256), 0, stream>>>(decay, log_g, p.H, p.N);
    return hipGetLastError();
}

// Scratch of the entry point that allocates nothing (lasp_fwd_noalloc): the segment states live in this
// array instead of a buffer the caller brings. Every device the library runs on holds its own copy, at
// its own address, until the process ends. The name below is a host-side stand-in, not a device address:
// host code uses the pointer static_scratch() returns, never the name.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch(void **ptr) {
    static std::mutex mu;
    static void *addr[64] = {};   // per device, filled on the first call with that device current
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(mu);
    if (!addr[dev]) {
        void *p = nullptr;
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return hipSuccess;
}

int cache_stride_for(int dtype, int tile, int ntiles, bool token, bool mixed_dims) {
    (void)token;       // both decay models have the pair kernel,
    (void)mixed_dims;  // and so do key and value dimensions that differ
    return (dtype == 1 && tile == 64 && ntiles % 2 == 0) ? 2 : 1;
}

// Tokens per kernel tile: 32 for float data, 64 for bfloat16 data, whatever the
// chunk (both divide every supported chunk length). 64-token bfloat16 tiles let two
// forward workgroups, or one backward workgroup with every tile it needs, live on a CU.
int tile_tokens(int dtype, int chunk, int D) {
    (void)chunk;
    (void)D;
    return dtype == 0 ? 32 : 64;
}

#define LASP_DISPATCH(FN, ARGS)                                                        \
    if (p.dk != p.dv) {   /* D = 128 kernels, the narrower of the two zero-padded */     \
        if (p.dtype == 0) {                                                            \
            if (p.dk == 64) return FN<float, 32, 128, 64, 128>(p, ARGS, stream, ke);      \
            return FN<float, 32, 128, 128, 64>(p, ARGS, stream, ke);                      \
        }                                                                              \
        if (p.dk == 64) return FN<bf16_t, 64, 128, 64, 128>(p, ARGS, stream, ke);         \
        return FN<bf16_t, 64, 128, 128, 64>(p, ARGS, stream, ke);                         \
    }                                                                                  \
    if (p.dtype == 0) {                                                                \
        if (p.D == 64) return FN<float, 32, 64>(p, ARGS, stream, ke);                     \
        return FN<float, 32, 128>(p, ARGS, stream, ke);                                    \
    }                                                                                  \
    if (p.D == 64) return FN<bf16_t, 64, 64>(p, ARGS, stream, ke);                         \
    return FN<bf16_t, 64, 128>(p, ARGS, stream, ke);

hipError_t launch_fwd(const Plan &p, const FwdArgs &a, hipStream_t stream, const KernelEvents *ke) { LASP_DISPATCH(run_fwd, a) }
hipError_t launch_bwd(const Plan &p, const BwdArgs &a, hipStream_t stream, const KernelEvents *ke) { LASP_DISPATCH(run_bwd, a) }

}  // namespace lasp
