// Device-side building blocks of the LASP kernels (gfx950 / CDNA4): MFMA operand
// fragments and their LDS fetch patterns, tile movement, LDS layouts, the two
// decay models, the Norm prologue and the small tile-level helpers the kernels
// in lasp_kernels.hip are assembled from. Device code only; included once.
#ifndef LASP_DEVICE_H
#define LASP_DEVICE_H

#include <hip/hip_runtime.h>

#include <type_traits>

namespace lasp {

typedef unsigned short bf16_t;  // storage type of bfloat16 data
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

#define DEVI __device__ __forceinline__

// Software pipelining of a product loop: the operand fragments of step s+1 are
// requested before the MFMAs of step s are issued, so that LDS latency is
// covered by matrix work of the same wave. `load(s)` returns the fragments of
// step s, `use(s, frags)` consumes them.
template <int N, typename Load, typename Use>
DEVI void pipelined(Load load, Use use) {
    // two steps ahead: with one or two waves per SIMD the LDS round trip is longer
    // than the matrix work of a single step
    auto cur = load(0);
    decltype(cur) nxt;
    if (N > 1) nxt = load(1);
#pragma unroll
    for (int s = 0; s < N; ++s) {
        decltype(cur) nn;
        if (s + 2 < N) nn = load(s + 2);
        use(s, cur);
        if (s + 1 < N) cur = nxt;
        if (s + 2 < N) nxt = nn;
    }
}
// The same for a long run of single-fragment steps with few registers: step i's fragment is requested
// AHEAD steps before it is used, so AHEAD fragments are in flight instead of whole multi-fragment steps.
template <int N, int AHEAD, typename Load, typename Use>
DEVI void pipelined_flat(Load load, Use use) {
    decltype(load(0)) ring[AHEAD];
#pragma unroll
    for (int i = 0; i < AHEAD && i < N; ++i) ring[i] = load(i);
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const auto cur = ring[i % AHEAD];
        if (i + AHEAD < N) ring[i % AHEAD] = load(i + AHEAD);
        use(i, cur);
    }
}
template <typename F>
struct FragPair {
    F a, b;
};

// Global access as (uniform base + compile-time bytes) + 32-bit per-lane byte
// offset: the form the hardware addresses with a scalar base register pair and
// one vector offset register, instead of a 64-bit address pair per access.
// STREAM: a non-temporal load. Used by the kernels that only sum over their input (local passes, state
// reduction): their reads then do not displace the previous kernel's still-dirty output from the
// last-level cache in the middle of a pure read stream (measured: these kernels 15-25 % faster, the step 2-3 %).
template <typename V, bool STREAM = false>
DEVI V gload(const void *base, unsigned lane_bytes) {
    if constexpr (STREAM) return __builtin_nontemporal_load((const V *)((const char *)base + lane_bytes));
    else return *(const V *)((const char *)base + lane_bytes);
}
template <typename V>
DEVI void gstore(void *base, unsigned lane_bytes, V v) { *(V *)((char *)base + lane_bytes) = v; }

// Lane coordinates inside a wave: id 0..63, r = row / column inside a 32-wide
// tile, h = which half of an MFMA's contraction step. A Lane is rebuilt from an
// opaque copy of the thread index at every phase of a kernel (fresh_lane), so
// the compiler derives the LDS/global lane offsets again where they are used
// instead of keeping dozens of loop-invariant address registers alive, which
// would spill; a spill reload queues behind the outstanding HBM prefetch.
struct Lane {
    int id, r, h;
    DEVI explicit Lane(int tid) : id(tid & 63), r(tid & 31), h((tid >> 5) & 1) {}
    // Row of accumulator register i (0..15) inside a 32x32 MFMA tile; the column is r.
    DEVI int acc_row(int i) const { return 8 * (i >> 2) + 4 * h + (i & 3); }
};
DEVI Lane fresh_lane() {
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return Lane(t);
}

// LDS layout of bfloat16 tiles with 128-element rows (256 bytes = all 64 banks):
// no padding; the 16-byte chunk c of row `row` is stored at chunk c ^ swz16(row).
// A row stride of exactly 128 elements selects this layout in the loaders below.
// It is conflict-free for 16 lanes reading one chunk of 16 consecutive rows, for
// the four-row by two-chunk blocks of a transposing read, and for whole-row stores.
constexpr int kSwzLd = 128;
DEVI int swz16(int row) { return ((row & 7) << 1) | ((row >> 3) & 1); }
// element offset of (row, col) in a tile with row stride ld
DEVI int lds_off(int ld, int row, int col) {
    return ld == kSwzLd ? row * kSwzLd + ((((col >> 3) ^ swz16(row))) << 3) + (col & 7) : row * ld + col;
}
template <typename T, int D>
constexpr int tile_ld() { return (sizeof(T) == 2 && D == 128) ? kSwzLd : D + (sizeof(T) == 2 ? 24 : 4); }

// ---------------------------------------------------------------------------
// Element traits: how MFMA operand fragments are fetched for each data type.
// A fragment is what one lane feeds to one MFMA: for a 32-row (or 32-column)
// operand block, lane (r, h) supplies row/column r and the h-th half of the
// KSTEP contraction indices of that MFMA.
//   ld_kc : contraction index contiguous in memory  X[(row0 + r) * ld + k]
//   ld_ks : contraction index strided in memory     X[k * ld + col0 + r]
//   ld_kp : contraction index contiguous, but taken in the permuted order in
//           which an accumulator tile enumerates its rows (sub-step m of the
//           32-wide block starting at kb), so that accumulator registers can be
//           the other operand.
// ---------------------------------------------------------------------------
template <typename T>
struct Elem;

template <>
struct Elem<float> {
    typedef float frag;
    static constexpr int KSTEP = 2;   // contraction extent of one MFMA
    static constexpr int NSUB = 16;   // MFMAs per 32-wide contraction block
    static constexpr int PAD = 4;     // elements of row padding in LDS tiles
    static DEVI f32x16 mfma(frag a, frag b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }
    static DEVI frag ld_kc(const Lane &ln, const float *X, int ld, int row0, int k0) { return X[(row0 + ln.r) * ld + k0 + ln.h]; }
    static DEVI frag ld_ks(const Lane &ln, const float *X, int ld, int k0, int col0) { return X[(k0 + ln.h) * ld + col0 + ln.r]; }
    // ld_kc from global memory: uniform tile pointer, row block row0, contraction step k0
    static DEVI frag ld_kc_g(const Lane &ln, const float *X, int ld, int row0, int k0) {
        return gload<float>(X + k0, ((row0 + ln.r) * ld + ln.h) * sizeof(float));
    }
    static DEVI frag ld_kp(const Lane &ln, const float *X, int ld, int row0, int kb, int m) {
        return X[(row0 + ln.r) * ld + kb + ln.acc_row(m)];
    }
    // accumulator tile -> fragment for sub-step m
    static DEVI frag from_acc(const f32x16 &t, int m) { return t[m]; }
    // multiply each contraction element k of the fragment by w[k]
    template <typename W>
    static DEVI frag scale(const Lane &ln, frag f, int k0, W w) { return f * w(k0 + ln.h); }
    // Elements per lane of one fragment, and the geometric form of a row weight:
    // every contraction element e of the fragment is multiplied by a * g[e].
    static constexpr int KH = 1;
    static DEVI frag scale_geo(frag f, float a, const float (&g)[8]) { return f * (a * g[0]); }
    // multiply contraction element k of the fragment of step k0 by tab[k] (tab in LDS)
    static DEVI frag scale_tab(const Lane &ln, frag f, const float *tab, int k0) { return f * tab[k0 + ln.h]; }
    // store 4 values of consecutive columns
    static DEVI void st4(float *p, float a, float b, float c, float d) { *(f32x4 *)p = f32x4{a, b, c, d}; }
    static DEVI void st1(float *p, float a) { *p = a; }
    static DEVI void gst4(float *base, unsigned lane_bytes, float a, float b, float c, float d) {
        gstore<f32x4>(base, lane_bytes, f32x4{a, b, c, d});
    }
    static DEVI void gst1(float *base, unsigned lane_bytes, float a) { gstore<float>(base, lane_bytes, a); }
    static DEVI float ld1(const float *p) { return *p; }
};

template <>
struct Elem<bf16_t> {
    typedef bf16x8 frag;
    static constexpr int KSTEP = 16;
    static constexpr int NSUB = 2;
    static constexpr int PAD = 8;   // 64-wide rows: stride 72 elements = 36 banks, an odd multiple of 4: the 16-byte reads of 16 consecutive rows and the 8-byte pieces of a transposing read over 4 rows fall on disjoint banks
    static DEVI f32x16 mfma(frag a, frag b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
    // row0 is a multiple of 16 and k0 a multiple of 16 wherever these are called.
    static DEVI frag ld_kc(const Lane &ln, const bf16_t *X, int ld, int row0, int k0) {
        if (ld == kSwzLd) {
            const int t = ln.h ^ swz16(ln.r);  // lane constant; chunk (k0/8 + h) ^ swz = (k0/8) ^ t since k0/8 is even
            return *(const bf16x8 *)(X + (row0 + ln.r) * kSwzLd + (((k0 >> 3) ^ t) << 3));
        }
        return *(const bf16x8 *)(X + (row0 + ln.r) * ld + k0 + 8 * ln.h);
    }
    static DEVI frag ld_kc_g(const Lane &ln, const bf16_t *X, int ld, int row0, int k0) {
        return gload<bf16x8>(X + k0, ((row0 + ln.r) * ld + 8 * ln.h) * sizeof(bf16_t));
    }
    // LDS only: two transposing reads (ds_read_b64_tr_b16). Within each group of
    // 16 lanes, lane i ends up with element (row e, column i) of the 4 x 16 block
    // whose rows the lanes addressed in 4-element pieces.
    static DEVI frag ld_ks(const Lane &ln, const bf16_t *X, int ld, int k0, int col0) {
        const int l = ln.id;
        const int l16 = l & 15;
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const bf16_t *plo, *phi;
        if (ld == kSwzLd) {
            const int rowl = 8 * ln.h + (l16 >> 2);                    // row inside the 16-row group (k0 % 16 == 0)
            const int c = (col0 >> 3) + 2 * ((l >> 4) & 1) + ((l16 & 3) >> 1);  // chunk of this lane's 8-byte piece
            const int e = 4 * (l16 & 1);                                // element inside the chunk
            plo = X + (k0 + rowl) * kSwzLd + ((c ^ swz16(rowl)) << 3) + e;
            phi = X + (k0 + rowl + 4) * kSwzLd + ((c ^ swz16(rowl + 4)) << 3) + e;
        } else {
            plo = X + (k0 + 8 * ln.h + (l16 >> 2)) * ld + col0 + 16 * ((l >> 4) & 1) + 4 * (l16 & 3);
            phi = plo + 4 * ld;
        }
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)plo);
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)phi);
        union { struct { s16x4 a, b; } s; bf16x8 v; } u;
        u.s.a = lo;
        u.s.b = hi;
        return u.v;
    }
    static DEVI frag ld_kp(const Lane &ln, const bf16_t *X, int ld, int row0, int kb, int m) {
        union { struct { bf16x4 a, b; } s; bf16x8 v; } u;
        if (ld == kSwzLd) {
            const int sw = swz16(ln.r), c = (kb >> 3) + 2 * m;
            const bf16_t *p = X + (row0 + ln.r) * kSwzLd + 4 * ln.h;
            u.s.a = *(const bf16x4 *)(p + ((c ^ sw) << 3));
            u.s.b = *(const bf16x4 *)(p + (((c + 1) ^ sw) << 3));
        } else {
            const bf16_t *p = X + (row0 + ln.r) * ld + kb + 16 * m + 4 * ln.h;
            u.s.a = *(const bf16x4 *)p;
            u.s.b = *(const bf16x4 *)(p + 8);
        }
        return u.v;
    }
    static DEVI frag from_acc(const f32x16 &t, int m) {
        f32x8 x;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = t[8 * m + e];
        return __builtin_convertvector(x, bf16x8);
    }
    template <typename W>
    static DEVI frag scale(const Lane &ln, frag f, int k0, W w) {
        f32x8 x = __builtin_convertvector(f, f32x8);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] *= w(k0 + 8 * ln.h + e);
        return __builtin_convertvector(x, bf16x8);
    }
    static constexpr int KH = 8;
    static DEVI frag scale_geo(frag f, float a, const float (&g)[8]) {
        f32x8 x = __builtin_convertvector(f, f32x8);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] *= a * g[e];
        return __builtin_convertvector(x, bf16x8);
    }
    static DEVI frag scale_tab(const Lane &ln, frag f, const float *tab, int k0) {
        const f32x4 *t = (const f32x4 *)(tab + k0 + 8 * ln.h);  // 16-byte aligned: tab is, k0 % 16 == 0
        const f32x4 lo = t[0], hi = t[1];
        f32x8 x = __builtin_convertvector(f, f32x8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] *= lo[e];
            x[4 + e] *= hi[e];
        }
        return __builtin_convertvector(x, bf16x8);
    }
    static DEVI void st4(bf16_t *p, float a, float b, float c, float d) {
        *(bf16x4 *)p = __builtin_convertvector(f32x4{a, b, c, d}, bf16x4);
    }
    static DEVI void st1(bf16_t *p, float a) {
        union { __bf16 b; bf16_t u; } c;
        c.b = (__bf16)a;
        *p = c.u;
    }
    static DEVI float ld1(const bf16_t *p) { return __uint_as_float(((unsigned)*p) << 16); }
    static DEVI void gst4(bf16_t *base, unsigned lane_bytes, float a, float b, float c, float d) {
        gstore<bf16x4>(base, lane_bytes, __builtin_convertvector(f32x4{a, b, c, d}, bf16x4));
    }
    static DEVI void gst1(bf16_t *base, unsigned lane_bytes, float a) { gstore<__bf16>(base, lane_bytes, (__bf16)a); }
};

// ---------------------------------------------------------------------------
// Tile movement: global -> registers -> LDS in 16-byte pieces. Splitting the
// two halves lets the next tile's loads fly while the current one is computed.
// ---------------------------------------------------------------------------
template <typename T, int ROWS, int COLS, int NT, bool STREAM = false>
struct TileMover {
    static constexpr int EPV = 16 / sizeof(T);          // elements per 16-byte piece
    static constexpr int VPR = COLS / EPV;              // pieces per row
    static constexpr int NV = ROWS * VPR / NT;          // pieces per thread
    static_assert(ROWS * VPR % NT == 0 && NT % VPR == 0, "tile must divide evenly over the workgroup");
    u32x4 r[NV];
    // Per-lane element offset of piece 0; piece i lies NT/VPR rows further down.
    static DEVI unsigned lane_off(int ld) { return (threadIdx.x / VPR) * ld + (threadIdx.x % VPR) * EPV; }
    DEVI void load(const T *g) {  // g: first element of the tile (uniform), row stride COLS
        const unsigned lo = lane_off(COLS) * sizeof(T);
#pragma unroll
        for (int i = 0; i < NV; ++i) r[i] = gload<u32x4, STREAM>(g + i * (NT / VPR) * COLS, lo);
    }
    // rows >= nrows are not touched in memory and read as zero (the last tile of a sub-sequence whose
    // length is not a multiple of the tile)
    DEVI void load(const T *g, int nrows) {
        if (nrows >= ROWS) return load(g);
        const unsigned lo = lane_off(COLS) * sizeof(T);
        const int row0 = threadIdx.x / VPR;
#pragma unroll
        for (int i = 0; i < NV; ++i)
            r[i] = row0 + i * (NT / VPR) < nrows ? gload<u32x4, STREAM>(g + i * (NT / VPR) * COLS, lo) : u32x4{0, 0, 0, 0};
    }
    // Tile of a tensor whose rows hold only W <= COLS elements (row stride W): columns >= W read as zero,
    // so a narrower key or value dimension rides through the COLS-wide kernels as zero padding.
    template <int W>
    DEVI void load_w(const T *g, int nrows) {
        if constexpr (W == COLS) {
            load(g, nrows);
        } else {
            static_assert(W < COLS && W % EPV == 0, "narrow rows are whole 16-byte pieces");
            const int row0 = threadIdx.x / VPR, chunk = threadIdx.x % VPR;
            const unsigned lo = (row0 * W + chunk * EPV) * sizeof(T);
            const bool col_ok = chunk * EPV < W;
#pragma unroll
            for (int i = 0; i < NV; ++i)
                r[i] = col_ok && row0 + i * (NT / VPR) < nrows ? gload<u32x4, STREAM>(g + i * (NT / VPR) * W, lo) : u32x4{0, 0, 0, 0};
        }
    }
    DEVI void store(T *s, int ld) const {
        if (sizeof(T) == 2 && ld == kSwzLd) {
            static_assert(sizeof(T) != 2 || COLS != 128 || (NT / VPR) % 16 == 0, "row step must keep row % 16");
            const int row = threadIdx.x / VPR, chunk = threadIdx.x % VPR;
            const unsigned lo = row * kSwzLd + ((chunk ^ swz16(row)) << 3);
#pragma unroll
            for (int i = 0; i < NV; ++i) *(u32x4 *)(s + i * (NT / VPR) * kSwzLd + lo) = r[i];
            return;
        }
        const unsigned lo = lane_off(ld);
#pragma unroll
        for (int i = 0; i < NV; ++i) *(u32x4 *)(s + i * (NT / VPR) * ld + lo) = r[i];
    }
};

// Sums across lanes without an LDS round trip.
// x + (the same value in the lane 32 further up or down): the two half-waves trade with one v_permlane32_swap.
DEVI float add_other_half(float x) {
    const auto t = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(t[0]) + __uint_as_float(t[1]);   // {lower, lower} + {upper, upper}
}
// Sum over groups of N consecutive lanes (N = 2 .. 16, a power of two, groups aligned), returned to all of
// them: a butterfly of data-parallel moves inside the 16-lane row (quad permutes for distance 1 and 2; once
// a quad holds one value, mirroring 8 and 16 lanes brings the other half's).
template <int N>
DEVI float group_sum(float x) {
    static_assert(N >= 1 && N <= 16 && (N & (N - 1)) == 0, "inside one row of 16 lanes");
    auto moved = [](float v, auto ctrl) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xf, 0xf, false));
    };
    using std::integral_constant;
    if constexpr (N >= 2) x += moved(x, integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
    if constexpr (N >= 4) x += moved(x, integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
    if constexpr (N >= 8) x += moved(x, integral_constant<int, 0x141>{});   // row_half_mirror
    if constexpr (N >= 16) x += moved(x, integral_constant<int, 0x140>{});  // row_mirror
    return x;
}

// ---------------------------------------------------------------------------
// Norm(.) of the normalised linear attention O = Norm((Q K^T (.) M) V) (Sec. 3.1, Eq. (2)),
// taken as the parameter-free root-mean-square normalisation of an output row:
//     y = o * rstd,  rstd = (mean_c o[c]^2 + eps)^(-1/2).
// Backward, applied to a tile of dY while it is still in registers on its way to
// LDS (the kernels then see dO as if it had been an input):
//     dO = rstd (dY - Y mean_c(dY[c] Y[c])).
// A row's pieces sit in COLS / EPV consecutive lanes of one wave, so the row mean
// is a butterfly over those lanes. NormTile holds what the prologue needs beside
// dY: the same pieces of Y and one rstd per piece row.
// ---------------------------------------------------------------------------
// W <= COLS: the rows in memory hold only W features (a value dimension narrower than the kernels');
// the mean runs over those W, the padding being zero.
template <typename T, int ROWS, int COLS, int NT, int W = COLS>
struct NormTile {
    typedef TileMover<T, ROWS, COLS, NT> TM;
    TM y;
    float rstd[TM::NV];
    // both pointers uniform: first element / first row of the tile; rows >= nrows (a short last tile) are
    // not touched in memory and count as y = 0, rstd = 0
    DEVI void load(const T *y_tile, const float *rstd_tile, int nrows = ROWS) {
        y.template load_w<W>(y_tile, nrows);
        const int row0 = threadIdx.x / TM::VPR;
        const unsigned lo = row0 * sizeof(float);
#pragma unroll
        for (int i = 0; i < TM::NV; ++i)
            rstd[i] = row0 + i * (NT / TM::VPR) < nrows ? gload<float>(rstd_tile + i * (NT / TM::VPR), lo) : 0.0f;
    }
    template <typename Mover>   // a TileMover of the same geometry (streaming or not)
    DEVI void apply(Mover &dy) const {
        static_assert(TM::VPR <= 32, "a row lies inside one half-wave");
        static_assert(Mover::NV == TM::NV && Mover::VPR == TM::VPR, "same tile geometry");
#pragma unroll
        for (int i = 0; i < TM::NV; ++i) {
            constexpr int E = TM::EPV;
            float a[E], b[E];
            if constexpr (sizeof(T) == 2) {
                union { u32x4 u; bf16x8 v; } ua, ub;
                ua.u = dy.r[i];
                ub.u = y.r[i];
                const f32x8 fa = __builtin_convertvector(ua.v, f32x8), fb = __builtin_convertvector(ub.v, f32x8);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    a[e] = fa[e];
                    b[e] = fb[e];
                }
            } else {
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    a[e] = __uint_as_float(dy.r[i][e]);
                    b[e] = __uint_as_float(y.r[i][e]);
                }
            }
            float p = 0.0f;
#pragma unroll
            for (int e = 0; e < E; ++e) p += a[e] * b[e];
            if constexpr (TM::VPR <= 16) {
                p = group_sum<TM::VPR>(p);
            } else {   // 32 lanes per row (float, 128 features): two rows of 16, then the neighbouring row
                p = group_sum<16>(p);
                p += __shfl_xor(p, 16, 64);
            }
            const float mean = p * (1.0f / W), rs = rstd[i];
#pragma unroll
            for (int e = 0; e < E; ++e) a[e] = rs * (a[e] - b[e] * mean);
            if constexpr (sizeof(T) == 2) {
                f32x8 f;
#pragma unroll
                for (int e = 0; e < E; ++e) f[e] = a[e];
                union { u32x4 u; bf16x8 v; } uo;
                uo.v = __builtin_convertvector(f, bf16x8);
                dy.r[i] = uo.u;
            } else {
#pragma unroll
                for (int e = 0; e < E; ++e) dy.r[i][e] = __float_as_uint(a[e]);
            }
        }
    }
};

// Row weights lambda^(CT-1-k) ("after": tokens after k in the tile) and lambda^(k+1)
// ("upto": 1-based position) for the KH consecutive tokens k_first .. k_first+KH-1 a
// lane holds in one fragment, as one table entry times a wave-uniform factor per element:
//   after: pw[CT-KH-k_first] * lambda^(KH-1-e)      upto: pw[k_first+1] * lambda^e
template <typename T>
struct GeoWeights {
    float after[8], upto[8];
    // (lam is the same in every lane; the factors are moved to scalar registers, where they cost no
    // vector registers for the length of the kernel)
    static DEVI float uniform(float x) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x))); }
    DEVI explicit GeoWeights(float lam) {
        const float l2f = (float)log2((double)lam);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            after[e] = e < Elem<T>::KH ? uniform(exp2f((float)(Elem<T>::KH - 1 - e) * l2f)) : 1.0f;
            upto[e] = e < Elem<T>::KH ? uniform(exp2f((float)e * l2f)) : 1.0f;
        }
    }
};
template <typename T, int CT>
DEVI typename Elem<T>::frag weigh_after(const Lane &ln, typename Elem<T>::frag f, int ks, const float *pw, const GeoWeights<T> &g) {
    const int k_first = ks * Elem<T>::KSTEP + Elem<T>::KH * ln.h;
    return Elem<T>::scale_geo(f, pw[CT - Elem<T>::KH - k_first], g.after);
}
template <typename T, int CT>
DEVI typename Elem<T>::frag weigh_upto(const Lane &ln, typename Elem<T>::frag f, int ks, const float *pw, const GeoWeights<T> &g) {
    const int k_first = ks * Elem<T>::KSTEP + Elem<T>::KH * ln.h;
    return Elem<T>::scale_geo(f, pw[k_first + 1], g.upto);
}

// lambda^n for n = 0..CT into LDS, evaluated in double so that the table adds
// no error of its own.
template <int CT>
DEVI void fill_pow_table(float *pw, float lam) {
    for (int i = threadIdx.x; i <= CT; i += blockDim.x) pw[i] = (float)exp2((double)i * log2((double)lam));
}

// ---------------------------------------------------------------------------
// Decay model of a tile of CT tokens (token indices 0-based inside the tile):
//   upto(i)      weight the state entering the tile carries at token i   (Lambda of Alg. 2)
//   after(j)     weight token j carries at the end of the tile           (lambda^C Lambda^-1)
//   whole()      weight the entering state carries at the end of the tile (lambda^C)
//   masked(x,i,j) x times the weight key j carries at query i, zero for j > i (mask M)
// FixedDecay: one lambda per head (Alg. 2 / Alg. 3 as printed); every weight is a
// power of lambda read from one table that serves all tiles.
// TokenDecay: a decay g_s per token (general recurrent form of App. A.4 with a
// scalar oscillation state); the weights are products of the g inside the tile,
// held as cumulative base-2 logarithms and rebuilt for every tile by fill().
// ---------------------------------------------------------------------------
template <typename T, int CT>
struct FixedDecay {
    static constexpr bool kToken = false;
    // Table in LDS: CT - 1 zeros, then lambda^0 .. lambda^(2 CT). pw points at lambda^0, so pw[d] is
    // lambda^d for 0 <= d <= 2 CT and ZERO for -(CT - 1) <= d < 0: the mask M (zero where the key comes after
    // the query) is a plain multiplication by pw[i - j], no compare and select. Exponents above CT serve the
    // kernel that reaches across a pair of tiles.
    static constexpr int kTableFloats = 3 * CT;
    const float *pw;
    GeoWeights<T> geo;
    DEVI FixedDecay(float *tab, float lam) : pw(tab + (CT - 1)), geo(lam) {
        const double l2 = log2((double)lam);   // evaluated in double so that the table adds no error of its own
        for (int i = threadIdx.x; i < kTableFloats; i += blockDim.x)
            tab[i] = i < CT - 1 ? 0.0f : (float)exp2((double)(i - (CT - 1)) * l2);
    }
    DEVI float upto(int i) const { return pw[i + 1]; }
    DEVI float after(int j) const { return pw[CT - 1 - j]; }
    DEVI float whole() const { return pw[CT]; }
    DEVI float masked(float x, int i, int j) const { return x * pw[i - j]; }
    DEVI typename Elem<T>::frag weigh_after(const Lane &ln, typename Elem<T>::frag f, int ks) const {
        return lasp::weigh_after<T, CT>(ln, f, ks, pw, geo);
    }
    DEVI typename Elem<T>::frag weigh_upto(const Lane &ln, typename Elem<T>::frag f, int ks) const {
        return lasp::weigh_upto<T, CT>(ln, f, ks, pw, geo);
    }
};

constexpr float kLog2e = 1.44269504088896340736f;

template <typename T, int CT>
struct TokenDecay {
    static constexpr bool kToken = true;
    static constexpr int PER = (CT + 63) / 64;  // tokens per lane of the wave that scans the tile
    static_assert(CT <= 128 && CT % PER == 0, "one wave scans a tile");
    // What fetch() brought for the wave that scans the tile: the raw log g of the lane's tokens and the number
    // of tokens the tile has. Nothing is computed from the loaded values before fill() needs them: an
    // instruction that touched them earlier would make the wave wait for the load right where it was issued,
    // in front of a tile's worth of products.
    struct LogG {
        float x[PER];
        int nvalid;
    };
    float *cum, *wu, *wa;  // LDS: cumulative log2 decay up to and including token i; 2^cum[i]; 2^(cum[CT-1]-cum[j])
    DEVI explicit TokenDecay(float *tab) : cum(tab), wu(tab + CT), wa(tab + 2 * CT) {}
    // log g of the tokens PER*l .. PER*l+PER-1 of the tile starting at `lg`, in lane l of wave 0 (other waves
    // load nothing). Tokens >= nvalid (past the end of the sub-sequence) are not read: their lanes fetch the
    // tile's first token instead and fill() counts them as log g = 0 (they do not decay the state).
    static DEVI LogG fetch(const float *lg, int nvalid = CT) {
        LogG v = {};
        v.nvalid = nvalid;
        if (threadIdx.x < 64) {
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int i = PER * threadIdx.x + e;
                v.x[e] = gload<float>(lg, (unsigned)((i < CT && i < nvalid) ? i : 0) * sizeof(float));
            }
        }
        return v;
    }
    // Inclusive prefix sum over the 64 lanes of a wave with data-parallel moves (no LDS round trips): four
    // shifts inside each row of 16 lanes, then the last lane of row 0 / 2 is added to row 1 / 3, then lane 31
    // to the upper half. Lanes a shift has no source for receive 0.
    static DEVI float wave_inclusive_scan(float x) {
        auto shifted = [](float v, auto ctrl, auto rows) {
            return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, decltype(rows)::value, 0xf, false));
        };
        using std::integral_constant;
        x += shifted(x, integral_constant<int, 0x111>{}, integral_constant<int, 0xf>{});   // row_shr:1
        x += shifted(x, integral_constant<int, 0x112>{}, integral_constant<int, 0xf>{});   // row_shr:2
        x += shifted(x, integral_constant<int, 0x114>{}, integral_constant<int, 0xf>{});   // row_shr:4
        x += shifted(x, integral_constant<int, 0x118>{}, integral_constant<int, 0xf>{});   // row_shr:8
        x += shifted(x, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{});   // row_bcast:15 into rows 1 and 3
        x += shifted(x, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{});   // row_bcast:31 into rows 2 and 3
        return x;
    }
    // Rebuilds the tables from the values fetch() returned. Every thread calls it between
    // the barrier that retires the previous tile and the one that publishes the next; the other waves
    // wait for the one that does the work, so it is kept short (register moves, the bare hardware exp2).
    // `base` (log2) is added to the exponents of both weight tables: a local pass that walks away from
    // the segment edge its weights refer to passes the decay between that edge and this tile, and never
    // has to rescale its accumulators. Returns the tile's total log2 decay (in the wave that fills; 0 elsewhere).
    DEVI float fill(const LogG &v, float base = 0.0f) const {
        float total = 0.0f;
        if (threadIdx.x < 64) {
            const int l = threadIdx.x;
            float c[PER];   // running sums of the lane's own tokens, log2
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int i = PER * l + e;
                const float x = (i < CT && i < v.nvalid) ? v.x[e] * kLog2e : 0.0f;
                c[e] = e ? c[e - 1] + x : x;
            }
            const float incl = wave_inclusive_scan(c[PER - 1]);  // inclusive scan of the lane totals
            total = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(incl), 63));  // lanes past the tile hold zeros
            const float before = incl - c[PER - 1];
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int i = PER * l + e;
                if (i < CT) {
                    const float ci = before + c[e];
                    cum[i] = ci;
                    wu[i] = __builtin_amdgcn_exp2f(base + ci);           // (below 2^-126: 0 instead of a denormal)
                    wa[i] = __builtin_amdgcn_exp2f(base + (total - ci));
                }
            }
        }
        return total;
    }
    DEVI float upto(int i) const { return wu[i]; }
    DEVI float after(int j) const { return wa[j]; }
    DEVI float whole() const { return wu[CT - 1]; }
    // (the bare hardware exp2: a weight below 2^-126 becomes 0 instead of a denormal, and the library
    // routine's range handling would cost four more instructions for every score element)
    DEVI float masked(float x, int i, int j) const { return i >= j ? x * __builtin_amdgcn_exp2f(cum[i] - cum[j]) : 0.0f; }
    DEVI typename Elem<T>::frag weigh_after(const Lane &ln, typename Elem<T>::frag f, int ks) const {
        return Elem<T>::scale_tab(ln, f, wa, ks * Elem<T>::KSTEP);
    }
    DEVI typename Elem<T>::frag weigh_upto(const Lane &ln, typename Elem<T>::frag f, int ks) const {
        return Elem<T>::scale_tab(ln, f, wu, ks * Elem<T>::KSTEP);
    }
};
template <bool TOKEN, typename T, int CT>
struct DecaySel {
    typedef FixedDecay<T, CT> type;
    // `decay` is lambda per head
    static DEVI type make(float *tab, const float *decay, int chain, int H) { return type(tab, decay[chain % H]); }
};
template <typename T, int CT>
struct DecaySel<true, T, CT> {
    typedef TokenDecay<T, CT> type;
    static DEVI type make(float *tab, const float *, int, int) { return type(tab); }
};

// floats of LDS behind the tiles of every kernel: decay tables, and one row of
// per-token partial sums per wave (backward walk with per-token decay)
template <int CT>
constexpr int table_floats() { return 3 * CT + 4 + 8 * CT; }

// Sum over this wave's 32 features of accT[feature][token] * X[token][feature] for the
// lane's token (accT: a transposed output tile in accumulator layout, X: the LDS tile
// with token rows starting at row0). Both half-waves end up with the full sum.
template <typename T>
DEVI float rowdot(const Lane &ln, const f32x16 &acc, const T *sX, int ld, int row0, int w) {
    float s = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        // the lane's four features of this register group are consecutive in the row (inside one 16-byte chunk)
        const T *p = sX + lds_off(ld, row0 + ln.r, 32 * w + 8 * q + 4 * ln.h);
        if constexpr (sizeof(T) == 2) {
            const f32x4 x = __builtin_convertvector(*(const bf16x4 *)p, f32x4);
#pragma unroll
            for (int e = 0; e < 4; ++e) s += acc[4 * q + e] * x[e];
        } else {
            const f32x4 x = *(const f32x4 *)p;
#pragma unroll
            for (int e = 0; e < 4; ++e) s += acc[4 * q + e] * x[e];
        }
    }
    return add_other_half(s);
}

// Load / store a wave's column block of a float state. In memory a state is [WK][WV] (row-major [a][c], row
// stride WV): the caller's states, the segment states in scratch and (in the data type) the state cache all
// hold only the real rows and columns; on chip the kernels work on the zero-padded [D][D] state in
// accumulator layout, st[ab][i] = S[32 ab + ln.acc_row(i)][32 w + ln.r]. Nothing outside [WK][WV] is touched
// in memory: padding is loaded as zero and never stored.
template <int D, int WK = D, int WV = D>
DEVI void state_load_w(const Lane &ln, f32x16 (&st)[D / 32], const float *g, int w) {
    const bool cols = 32 * w < WV;   // (wave-uniform) this wave's column block holds real columns
    const unsigned lo = (4 * ln.h * WV + 32 * w + ln.r) * sizeof(float);
#pragma unroll
    for (int ab = 0; ab < D / 32; ++ab)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            st[ab][i] = (ab < WK / 32 && cols) ? gload<float>(g + (32 * ab + 8 * (i >> 2) + (i & 3)) * WV, lo) : 0.0f;
}
// The same state in the other orientation: st[cb][i] = S[32 w + ln.r][32 cb + ln.acc_row(i)] (the wave owns 32 rows).
template <int D, int WK = D, int WV = D>
DEVI void state_load_t_w(const Lane &ln, f32x16 (&st)[D / 32], const float *g, int w) {
    const bool rows = 32 * w < WK;
    const unsigned lo = ((32 * w + ln.r) * WV + 4 * ln.h) * sizeof(float);
#pragma unroll
    for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 x = (cb < WV / 32 && rows) ? gload<f32x4>(g + 32 * cb + 8 * q, lo) : f32x4{0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 4; ++e) st[cb][4 * q + e] = x[e];
        }
}
template <int D, int WK = D, int WV = D>
DEVI void state_store_w(const Lane &ln, const f32x16 (&st)[D / 32], float *g, int w) {
    if constexpr (WV < D) {
        if (32 * w >= WV) return;
    }
    const unsigned lo = (4 * ln.h * WV + 32 * w + ln.r) * sizeof(float);
#pragma unroll
    for (int ab = 0; ab < WK / 32; ++ab)
#pragma unroll
        for (int i = 0; i < 16; ++i) gstore<float>(g + (32 * ab + 8 * (i >> 2) + (i & 3)) * WV, lo, st[ab][i]);
}

// Masked score tile (Alg. 2 / Alg. 3 mask M): the wave holds the transposed
// 32x32 block ST[j][i] = sum_d A[j][d] B[i][d] in accumulator layout (row = key j,
// column = query i), multiplies by lambda^(i-j) for i >= j (zero above the
// diagonal) and writes it as P[i][j] so that four consecutive keys land in one
// store.
template <typename T, int LDP, typename DK>
DEVI void store_masked_scores(const Lane &ln, T *sP, const f32x16 &acc, int jb, int ib, const DK &dec) {
    const int iq = 32 * ib + ln.r;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int j0 = 32 * jb + 8 * g + 4 * ln.h;
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = dec.masked(acc[4 * g + e], iq, j0 + e);
        Elem<T>::st4(sP + iq * LDP + j0, x[0], x[1], x[2], x[3]);
    }
}

// ST[jb][ib] = A[jb] B[ib]^T over the feature dimension (both operands have the
// contraction index contiguous), for every lower-triangular block assigned to
// this wave; result masked and stored to sP.
template <typename T, int CT, int D, int LDD, int LDP, typename DK>
DEVI void masked_scores(const Lane &ln, T *sP, const T *sA, const T *sB, const DK &dec, int w) {
    using E = Elem<T>;
    constexpr int NB = CT / 32, NW = D / 32;
    int idx = 0;
#pragma unroll
    for (int ib = 0; ib < NB; ++ib)
#pragma unroll
        for (int jb = 0; jb <= ib; ++jb, ++idx) {
            if (idx % NW != w) continue;
            f32x16 acc = {0};
#pragma unroll
            for (int k0 = 0; k0 < D; k0 += E::KSTEP)
                acc = E::mfma(E::ld_kc(ln, sA, LDD, 32 * jb, k0), E::ld_kc(ln, sB, LDD, 32 * ib, k0), acc);
            store_masked_scores<T, LDP>(ln, sP, acc, jb, ib, dec);
        }
}

// Write one 32x32 accumulator tile holding the TRANSPOSE of an output block:
// accumulator row = feature column 32 w + ln.acc_row(i), accumulator column
// (lane_r) = token row0 + lane_r. Each lane owns four consecutive features of
// its token per register group, so it stores them as one 8- or 16-byte piece.
// W <= D: the tensor's rows hold only W features (row stride W); waves whose column block lies
// beyond them hold padding and store nothing.
// The two-byte form of such a tile, ready to store. The lane's four features of a register group are 8
// bytes, and a store instruction of 8-byte pieces would leave 16 bytes in each of 32 rows. Two exchanges
// between lanes widen that:
//   - The two half-waves hold neighbouring features of the same token, so they trade register groups
//     (v_permlane32_swap: lanes 32..63 of the first operand against lanes 0..31 of the second): every
//     lane then holds two 16-byte pieces of its token, features 16 p + 8 h .. + 7 (p = 0, 1).
//   - Lanes 16 apart hold the same pieces of tokens 16 apart, so piece 1 of the lower 16 tokens is traded
//     against piece 0 of the upper 16 (v_permlane16_swap: odd 16-lane rows of the first operand against
//     even rows of the second): v[0] then holds all four pieces (64 contiguous bytes) of tokens 0..15,
//     v[1] those of tokens 16..31. A store instruction writes 16 rows of 64 bytes, not 32 rows of 32:
//     half the memory requests for the same bytes.
// After both, lane l holds in v[j] the features 16 ((l >> 4) & 1) + 8 (l >> 5) .. + 7 of token 16 j + (l & 15)
// (features relative to the wave's 32-feature block, tokens relative to the tile's 32-token block).
struct PackedTile {
    u32x4 v[2];
};
DEVI PackedTile pack_out_tile_t(const f32x16 &acc) {
    u32x2 d[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        union { bf16x4 v; u32x2 u; } pk;
        pk.v = __builtin_convertvector(f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]}, bf16x4);
        d[q] = pk.u;
    }
    u32x4 piece[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const u32x2 s0 = __builtin_amdgcn_permlane32_swap(d[2 * p][0], d[2 * p + 1][0], false, false);
        const u32x2 s1 = __builtin_amdgcn_permlane32_swap(d[2 * p][1], d[2 * p + 1][1], false, false);
        piece[p] = u32x4{s0[0], s1[0], s0[1], s1[1]};
    }
    PackedTile t;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const u32x2 x = __builtin_amdgcn_permlane16_swap(piece[0][e], piece[1][e], false, false);
        t.v[0][e] = x[0];
        t.v[1][e] = x[1];
    }
    return t;
}
// g: first element of the tile (uniform); rows hold W two-byte elements; the wave's block starts at feature 32 w
template <typename T, int W>
DEVI void store_packed_tile_t(const Lane &ln, T *g, const PackedTile &t, int row0, int w, int nrows = 1 << 30) {
    static_assert(sizeof(T) == 2, "two-byte elements");
    const int tok = ln.id & 15, feat = 32 * w + 16 * ((ln.id >> 4) & 1) + 8 * (ln.id >> 5);
    const unsigned lo = (tok * W + feat) * sizeof(T);
#pragma unroll
    for (int j = 0; j < 2; ++j)
        if (row0 + 16 * j + tok < nrows) gstore<u32x4>(g + (row0 + 16 * j) * W, lo, t.v[j]);
}

template <typename T, int D, int W = D>
DEVI void store_out_tile_t(const Lane &ln, T *g, const f32x16 &acc, int row0, int w, int nrows = 1 << 30) {
    if constexpr (W < D) {
        if (32 * w >= W) return;
    }
    if constexpr (sizeof(T) == 2) {
        store_packed_tile_t<T, W>(ln, g, pack_out_tile_t(acc), row0, w, nrows);
    } else {
        const unsigned lo = (ln.r * W + 32 * w + 4 * ln.h) * sizeof(T);
        if (row0 + ln.r >= nrows) return;  // token past the end of the sub-sequence
#pragma unroll
        for (int q = 0; q < 4; ++q)
            Elem<T>::gst4(g + row0 * W + 8 * q, lo, acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    }
}

// Store a wave's column block of the state into the cache tile g ([a][c], [WK][WV] real rows and columns,
// row stride WV). Accumulator layout gives each lane four consecutive a for one c,
// the wrong way round for wide stores, so for bfloat16 the wave transposes one
// 32x32 block at a time through a private slice of an idle LDS buffer (written
// [c][a], read back with transposing reads) and stores 16 bytes per lane:
// 64-byte row segments instead of single elements. Other types store element
// by element. The LDS slice is only touched by this wave (LDS operations of one
// wave execute in order); the caller's next barrier orders it against later use.
// Waves whose column block is padding (32 w >= WV) and row blocks of padding (ab >= WK / 32) store nothing.
template <typename T, int CT, int D, int WK = D, int WV = D>
DEVI void cache_store(const Lane &ln, T *g, const f32x16 (&st)[D / 32], T *idle_lds, int w) {
    using E = Elem<T>;
    constexpr int LDS_ROW = 36;  // 32 a + 4 pad elements: 8-byte aligned rows, staggered banks
    constexpr bool STAGED = sizeof(T) == 2 && (D / 32) * 32 * LDS_ROW <= CT * (CT + E::PAD);
    if constexpr (WV < D) {
        if (32 * w >= WV) return;
    }
    if constexpr (STAGED) {
        T *R = idle_lds + w * 32 * LDS_ROW;
        const int l = ln.id, bl = l >> 4, i = l & 15;
        const unsigned glo = (i * WV + 32 * w + 8 * bl) * sizeof(T);
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
#pragma unroll
        for (int ab = 0; ab < WK / 32; ++ab) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                E::st4(R + ln.r * LDS_ROW + 8 * q + 4 * ln.h, st[ab][4 * q], st[ab][4 * q + 1], st[ab][4 * q + 2],
                       st[ab][4 * q + 3]);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const T *p = R + (8 * bl + (i >> 2)) * LDS_ROW + 16 * it + 4 * (i & 3);
                union { struct { s16x4 a, b; } s; u32x4 v; } u;
                u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
                u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * LDS_ROW));
                gstore<u32x4>(g + (32 * ab + 16 * it) * WV, glo, u.v);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    } else {
        const unsigned slo = (4 * ln.h * WV + 32 * w + ln.r) * sizeof(T);
#pragma unroll
        for (int ab = 0; ab < WK / 32; ++ab)
#pragma unroll
            for (int i = 0; i < 16; ++i) E::gst1(g + (32 * ab + 8 * (i >> 2) + (i & 3)) * WV, slo, st[ab][i]);
    }
}

}  // namespace lasp
#endif  // LASP_DEVICE_H
