/*
 * lasp.h -- C ABI of the MI355X (gfx950) hot path of LASP, arxiv 2404.02882:
 * causal linear attention with per-head decay, computed chunk by chunk with a
 * carried d x d KV state (forward) and a carried dKV state (backward).
 *
 * One call processes one sub-sequence of N tokens for all B*H heads. A longer
 * sequence is processed as successive calls: forward in order, handing kv_out
 * of one call to the next as kv_in; backward in reverse order, handing dkv_in
 * of one call to the previous as dkv_out. This loop is the paper's ring of
 * ranks (Alg. 2 Recv/Send of KV, Alg. 3 Recv/Send of dKV) folded onto one GPU:
 * the messages are these state buffers.
 *
 * Common conventions
 *   - Every pointer is a DEVICE pointer owned by the caller. The library never
 *     allocates, frees or synchronises: work is enqueued on `hip_stream`
 *     (a hipStream_t; NULL = the default stream) and the call returns at once.
 *   - q, k, v, out, dout, dq, dk, dv: [B][H][N][D], row-major, one token row is
 *     D contiguous elements of `dtype` (LASP_F32: float, LASP_BF16: bfloat16).
 *   - kv_in, kv_out, dkv_out, dkv_in: [B][H][D][D] float, state[a][c] with a the
 *     key/query feature and c the value feature (KV = sum k[a] v[c]).
 *     (With lasp_shape.Dv set, value-side tensors have Dv columns and states are
 *     [D][Dv]; with lasp_shape.kv_heads set, k, v, dk, dv have kv_heads heads.)
 *   - decay: [H] float on the device, lambda_h in (0, 1], shared over the
 *     batch; lambda = 1 is ordinary linear attention (Sec. 3.2). It is not
 *     learnable, so no gradient is produced for it.
 *   - Every function returns a lasp_status; nothing throws or aborts. All
 *     argument checks run on the host before anything is launched.
 *   - Every buffer is 16-byte aligned (the kernels move 16-byte pieces).
 *   - Outputs must not alias inputs or each other. Calls that share a scratch
 *     or state_cache buffer must be ordered on one stream.
 */
#ifndef LASP_H
#define LASP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LASP_OK = 0,
    LASP_ERR_NULL = 1,      /* a required pointer is NULL */
    LASP_ERR_SHAPE = 2,     /* B,H,N <= 0; D or Dv not 64/128; chunk not 64/128/256; bad segments or kv_heads */
    LASP_ERR_DTYPE = 3,     /* dtype is neither LASP_F32 nor LASP_BF16 */
    LASP_ERR_DECAY = 4,     /* lasp_check_decay: a value outside (0, 1] or not finite */
    LASP_ERR_WORKSPACE = 5, /* scratch missing or smaller than lasp_scratch_bytes() */
    LASP_ERR_ALIAS = 6,     /* an output buffer overlaps an input or another output */
    LASP_ERR_HIP = 7,       /* the HIP runtime refused a launch */
    LASP_ERR_ALIGN = 8      /* a buffer is not 16-byte aligned */
} lasp_status;

typedef enum { LASP_F32 = 0, LASP_BF16 = 1 } lasp_dtype;

/*
 * Problem shape of one call.
 *   N        tokens in this sub-sequence (the paper's per-rank length N/T), any
 *            positive number. When N is not a multiple of lasp_tile_tokens() the
 *            last tile is short; the per-token-decay kernels handle that, so
 *            lasp_fwd / lasp_bwd then run those with log g = log(lambda) filled in
 *            by the library (about 10 % slower, more scratch).
 *   chunk    the chunk length C of Alg. 2 / Alg. 3: 64, 128 or 256. It is checked
 *            and otherwise NOT USED: the kernels always walk the sub-sequence in
 *            tiles of lasp_tile_tokens() tokens, which divide every allowed chunk.
 *            The results are those of any chunk length, because the state update
 *            of Sec. 3.2 composes over consecutive tiles.
 *   kv_heads 0 or H: every query head has its own key/value head. Otherwise a
 *            divisor of H: k, v (and dk, dv) are [B][kv_heads][N][D] and the
 *            H / kv_heads consecutive query heads of a group share one of them
 *            (multi-query / grouped-query heads, which the method is indifferent
 *            to: Sec. 1). States, decays and everything indexed by head stay per
 *            QUERY head. The backward pass then needs scratch for dK, dV per query
 *            head (two token tensors), summed over each group at the end.
 *   Dv       0 or D: queries, keys and values share the head dimension D. Otherwise
 *            the value dimension d_v (64 or 128) while D is the key dimension d_k:
 *            q, k, dq, dk are [..][N][D], v, out, dout, dv are [..][N][Dv], and
 *            every state (kv_in, kv_out, dkv_out, dkv_in) is [B][H][D][Dv], rows
 *            indexed by the key feature. The kernels run at max(D, Dv) with the
 *            narrower of the two zero-padded on chip; memory traffic, scratch and
 *            the state cache follow the real sizes. The fused
 *            Norm then runs over the Dv value features. Not offered for the
 *            bidirectional calls.
 *   segments 0 = chosen by the library. Otherwise the number of independent
 *            segments each head's sub-sequence is cut into so that B*H*segments
 *            workgroups fill the chip (1 <= segments <= ceil(N / tile)).
 */
typedef struct {
    int32_t B, H, N, D, chunk;
    int32_t dtype;    /* lasp_dtype */
    int32_t segments; /* 0 = auto */
    int32_t kv_heads; /* 0 = H */
    int32_t Dv;       /* 0 = D */
} lasp_shape;

int lasp_version(void);
const char *lasp_status_str(int status);

/* Validates a shape exactly as lasp_fwd / lasp_bwd do. Host only. */
int lasp_check_shape(const lasp_shape *shape);

/* Validates a HOST copy of the decay vector: every value finite and in (0, 1]. */
int lasp_check_decay(const float *decay_host, int32_t H);

/* Tokens per kernel tile for this shape (divides chunk); 0 on an invalid shape. */
int32_t lasp_tile_tokens(const lasp_shape *shape);

/* Segments per head the forward pass will use for this shape (the backward pass
 * may choose fewer when `segments` is 0); 0 on an invalid shape. */
int32_t lasp_num_segments(const lasp_shape *shape);

/*
 * Bytes of the state cache: the states KV_{t-1} that tiles start from, written
 * by lasp_fwd and read by lasp_bwd for dQ_inter (the paper caches the state a
 * rank receives, Alg. 2 "save KV_{t-1}", Sec. 3.4; this build caches one state
 * per tile, or one per two tiles where the backward kernel reaches the other
 * tile from its neighbour's state, so that the backward pass never reruns the
 * forward recurrence).
 * The layout is private to the library; slot 0 is kv_in. Stored in `dtype`.
 * 0 on an invalid shape.
 */
size_t lasp_state_cache_bytes(const lasp_shape *shape);

/*
 * Bytes of scratch both lasp_fwd and lasp_bwd need: one float [D][Dv] state per
 * head per segment. Contents are overwritten by every call. 0 on an invalid shape.
 */
size_t lasp_scratch_bytes(const lasp_shape *shape);

/*
 * Forward (Alg. 2 without the projections and with Recv/Send replaced by
 * kv_in/kv_out). For every head and token s = 1..N of this sub-sequence:
 *     out_s  = sum_{i<=s} lambda^(s-i) (q_s . k_i) v_i  +  lambda^s kv_in^T q_s
 *     kv_out = lambda^N kv_in + sum_i lambda^(N-i) k_i v_i^T
 * computed per tile as O = [(Q K^T) (.) M] V + Lambda Q KV_{t-1} and
 * KV_t = lambda^C KV_{t-1} + (lambda^C Lambda^-1 K)^T V.
 *
 *   kv_in        NULL = zeros (first sub-sequence, Alg. 2 "KV = 0").
 *   out, kv_out  required.
 *   state_cache  NULL = forward only, nothing cached; else at least
 *                lasp_state_cache_bytes() bytes, to be passed to lasp_bwd.
 *   scratch      at least lasp_scratch_bytes() bytes (scratch_bytes = its size).
 */
int lasp_fwd(const lasp_shape *shape, const void *q, const void *k, const void *v,
             const float *kv_in, const float *decay, void *out, float *kv_out,
             void *state_cache, void *scratch, size_t scratch_bytes, void *hip_stream);

/*
 * lasp_fwd for callers that cannot allocate device memory or must not pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc. Same computation, same kernels and bit-identical results;
 * the scratch (segment states) is a fixed array inside the library instead of a
 * caller's buffer. The call allocates and frees nothing and does not synchronise.
 *   - The array holds lasp_noalloc_scratch_limit() bytes (32 MiB) on every
 *     device the library is used on, until the process ends. A shape whose
 *     lasp_scratch_bytes() exceeds it is rejected with LASP_ERR_WORKSPACE before
 *     anything is launched (lower `segments`, or use lasp_fwd).
 *   - All calls on one device share that array: calls that overlap in time on one
 *     device (different streams, or threads) race. Order them on one stream.
 *     Nothing in it needs clearing between calls: every slot a call reads it has
 *     written first.
 *   - The first call on a device resolves the array's address (one host-side
 *     look-up, no allocation); make that call outside a graph capture.
 * Arguments and statuses otherwise as for lasp_fwd.
 */
int lasp_fwd_noalloc(const lasp_shape *shape, const void *q, const void *k, const void *v,
                     const float *kv_in, const float *decay, void *out, float *kv_out,
                     void *state_cache, void *hip_stream);
size_t lasp_noalloc_scratch_limit(void);

/*
 * Backward (Alg. 3 with Recv/Send replaced by dkv_out/dkv_in). Gradients of
 *     L = sum(out * dout) + sum(kv_out * dkv_out):
 *     dq_s = kv_s do_s,  dk_s = dkv_s v_s,  dv_s = dkv_s^T k_s,
 *     dkv_s = sum_{i>=s} lambda^(i-s) q_i do_i^T + lambda^(N-s) dkv_out,
 *     dkv_in = lambda^N dkv_out + sum_s lambda^s q_s do_s^T   (gradient w.r.t. kv_in)
 * computed per tile as in Alg. 3 (intra parts from the masked S and dS, inter
 * parts from the cached KV_{t-1} and the carried dKV).
 *
 *   dkv_out      NULL = zeros (last sub-sequence, Alg. 3 "dKV = 0").
 *   state_cache  the buffer the matching lasp_fwd call filled (same shape, same
 *                inputs, same kv_in), or NULL = recompute: the paper's alternative
 *                to caching (Sec. 3.4, "KV state caching" on / off). The call then
 *                rebuilds the states first, from k, v and kv_in, with the forward
 *                kernels reduced to their states (Alg. 2 without the outputs),
 *                into the tail of `scratch`, which must then hold at least
 *                lasp_bwd_recompute_scratch_bytes(). Nothing has to be kept between
 *                the forward and the backward pass but kv_in; the price is one more
 *                pass over k, v.
 *   kv_in        the state the sub-sequence started from (what lasp_fwd was given;
 *                NULL = zeros). Read only when state_cache is NULL: the cache's first
 *                slot already holds it.
 *   dq, dk, dv, dkv_in  required.
 */
int lasp_bwd(const lasp_shape *shape, const void *q, const void *k, const void *v,
             const void *dout, const float *kv_in, const float *dkv_out, const float *decay,
             const void *state_cache, void *dq, void *dk, void *dv, float *dkv_in,
             void *scratch, size_t scratch_bytes, void *hip_stream);

/*
 * Bytes of scratch lasp_bwd (and lasp_bwd_norm) needs when it is given no state
 * cache: lasp_scratch_bytes() rounded up to 256, plus lasp_state_cache_bytes().
 * 0 on an invalid shape.
 */
size_t lasp_bwd_recompute_scratch_bytes(const lasp_shape *shape);

/*
 * ---- Per-token decay -------------------------------------------------------
 * The same path for the general recurrent form of App. A.4, m_t = o_t m_{t-1} +
 * e_t i_t^T, with a scalar oscillation state o_t = g_t per head and token (Table 6:
 * the TNL/RetNet row is the constant g_t = lambda; a decay that depends on the
 * token is the scalar case of the GLA/GateLoop and Mamba rows):
 *     kv_s = g_s kv_{s-1} + k_s v_s^T,     out_s = kv_s^T q_s,
 * i.e. with W(i,s) = g_{i+1} ... g_s (empty product = 1)
 *     out_s  = sum_{i<=s} W(i,s) (q_s . k_i) v_i + W(0,s) kv_in^T q_s
 *     kv_out = W(0,N) kv_in + sum_i W(i,N) k_i v_i^T.
 * Per tile this is Alg. 2 / Alg. 3 with M_ij = W(j,i), Lambda = diag{W(0,i)},
 * lambda^C Lambda^-1 = diag{W(j,C)}, lambda^C = W(0,C).
 *
 *   log_g   DEVICE float [B][H][N]: natural logarithm of g, finite and <= 0. The
 *           library cannot inspect device memory; lasp_check_log_decay validates a
 *           host copy. Values > 0 or non-finite give undefined numbers (never a
 *           fault).
 *   dlog_g  DEVICE float [B][H][N]: gradient of the loss w.r.t. log g_s,
 *               dlog_g_s = <dkv_out, kv_out> + sum_{t>=s} (q_t . dq_t - k_t . dk_t).
 *   kv_out  (backward) the state the matching lasp_gated_fwd returned; required
 *           when dkv_out is given, ignored otherwise.
 *   kv_in   (backward) as for lasp_bwd: read only when state_cache is NULL
 *           (recompute; scratch of lasp_gated_bwd_recompute_scratch_bytes()).
 * Everything else (layouts, states, state_cache, scratch, stream, status codes,
 * aliasing rules) is as for lasp_fwd / lasp_bwd, with the sizes from the
 * lasp_gated_* size functions.
 */
int lasp_check_log_decay(const float *log_g_host, int64_t n);
size_t lasp_gated_state_cache_bytes(const lasp_shape *shape);
size_t lasp_gated_scratch_bytes(const lasp_shape *shape);
size_t lasp_gated_bwd_recompute_scratch_bytes(const lasp_shape *shape);
int lasp_gated_fwd(const lasp_shape *shape, const void *q, const void *k, const void *v,
                   const float *log_g, const float *kv_in, void *out, float *kv_out,
                   void *state_cache, void *scratch, size_t scratch_bytes, void *hip_stream);
int lasp_gated_bwd(const lasp_shape *shape, const void *q, const void *k, const void *v,
                   const void *dout, const float *log_g, const float *kv_in, const float *kv_out,
                   const float *dkv_out, const void *state_cache, void *dq, void *dk, void *dv,
                   float *dlog_g, float *dkv_in, void *scratch, size_t scratch_bytes,
                   void *hip_stream);

/*
 * ---- Normalised output ------------------------------------------------------
 * O = Norm((Q K^T (.) M) V) (Sec. 3.1, Eq. (2); Sec. 3.2 drops
 * the Norm only to shorten its derivation). The paper does not spell Norm out;
 * here it is the parameter-free root-mean-square normalisation of every output
 * row over the head dimension,
 *     y_s = o_s * rstd_s,   rstd_s = (mean_c o_s[c]^2 + eps)^(-1/2),
 * fused into the forward kernel's epilogue (o never goes to memory) and into
 * the backward kernels' prologue:  do_s = rstd_s (dy_s - y_s mean_c(dy_s[c] y_s[c])).
 * lasp_fwd / lasp_bwd semantics otherwise (one lambda per head; the per-token
 * decay has its own pair below).
 *
 *   eps     >= 0, finite (LASP_ERR_SHAPE otherwise).
 *   out     forward: the NORMALISED output y, [B][H][N][D] in `dtype`; backward:
 *           the same buffer, as input.
 *   rstd    DEVICE float [B][H][N]: written by lasp_fwd_norm, read by lasp_bwd_norm.
 *   dout    backward: gradient w.r.t. the normalised output y.
 *   kv_in, state_cache (backward): as for lasp_bwd, NULL cache = recompute.
 */
int lasp_fwd_norm(const lasp_shape *shape, const void *q, const void *k, const void *v,
                  const float *kv_in, const float *decay, float eps, void *out, float *rstd,
                  float *kv_out, void *state_cache, void *scratch, size_t scratch_bytes,
                  void *hip_stream);
int lasp_bwd_norm(const lasp_shape *shape, const void *q, const void *k, const void *v,
                  const void *out, const float *rstd, const void *dout, const float *kv_in,
                  const float *dkv_out, const float *decay, const void *state_cache, void *dq,
                  void *dk, void *dv, float *dkv_in, void *scratch, size_t scratch_bytes,
                  void *hip_stream);

/*
 * Per-token decay and normalised output together: arguments as in
 * lasp_gated_fwd / lasp_gated_bwd plus eps, rstd and (backward) the normalised
 * output, with the meaning they have in lasp_fwd_norm / lasp_bwd_norm; dout is
 * the gradient w.r.t. the normalised output.
 */
int lasp_gated_fwd_norm(const lasp_shape *shape, const void *q, const void *k, const void *v,
                        const float *log_g, const float *kv_in, float eps, void *out, float *rstd,
                        float *kv_out, void *state_cache, void *scratch, size_t scratch_bytes,
                        void *hip_stream);
int lasp_gated_bwd_norm(const lasp_shape *shape, const void *q, const void *k, const void *v,
                        const void *out, const float *rstd, const void *dout, const float *log_g,
                        const float *kv_in, const float *kv_out, const float *dkv_out,
                        const void *state_cache, void *dq, void *dk, void *dv, float *dlog_g,
                        float *dkv_in, void *scratch, size_t scratch_bytes, void *hip_stream);

/*
 * ---- Bidirectional (unmasked) attention ---------------------------------------
 * Without the causal mask the attention of Sec. 3.1 is O = (Q K^T) V, which
 * associativity turns into the right-product form O = Q (K^T V) of Eq. (3)
 * (here without the Norm). There is no decay and no order among the tokens:
 * the d x d state is the plain sum KV = sum_s k_s v_s^T over EVERY token of the
 * sequence, so sub-sequences do not form a chain. Each adds its tokens to the
 * state (on several devices: one sum of a [B][H][D][D] float tensor across
 * them), and only then does any of them compute its outputs:
 *     forward : KV  = sum_s k_s v_s^T     (lasp_bidir_state on K, V, once per sub-sequence)
 *               O   = Q KV                (lasp_bidir_fwd)
 *     backward: dKV = sum_s q_s do_s^T    (lasp_bidir_state on Q, dO, once per sub-sequence)
 *               dQ  = dO KV^T,  dK = V dKV^T,  dV = K dKV    (lasp_bidir_bwd)
 * The paper states the formula only; the split into these calls, and summing
 * the state across sub-sequences instead of handing it round a ring, are this
 * library's reading of it.
 *
 * Shapes as in lasp_shape with kv_heads 0 or H (LASP_ERR_SHAPE otherwise);
 * `chunk` must be a valid chunk length but has no effect; any N >= 1;
 * `segments`: 0 = automatic, else the number of partial sums per head of the
 * state reduction (1 <= segments <= ceil(N / tile)). Token tensors
 * [B][H][N][D] in `dtype`, states [B][H][D][D] float with rows indexed by the
 * FIRST factor's feature (k, resp. q), all in DEVICE memory, 16-byte aligned,
 * outputs not overlapping inputs or each other. Statuses and asynchrony as for
 * lasp_fwd. Products run on MFMA in `dtype` with fp32 accumulation; a state is
 * rounded to `dtype` where it enters a product.
 */
/* Bytes of scratch lasp_bidir_state needs (partial sums); 0 on an invalid shape. */
size_t lasp_bidir_scratch_bytes(const lasp_shape *shape);
/*
 * state (+)= sum over this sub-sequence's tokens s of x_s y_s^T, per head.
 *   accumulate  0: state is overwritten; otherwise the sum is added to it (the
 *               second and later sub-sequences, or a state received from elsewhere).
 * Partial sums are added in a fixed order: bit-reproducible.
 */
int lasp_bidir_state(const lasp_shape *shape, const void *x, const void *y, float *state,
                     int32_t accumulate, void *scratch, size_t scratch_bytes, void *hip_stream);
/* out = q kv for every head: [N][D] x [D][D]. */
int lasp_bidir_fwd(const lasp_shape *shape, const void *q, const float *kv, void *out,
                   void *hip_stream);
/* dq = dout kv^T, dk = v dkv^T, dv = k dkv (kv, dkv: the complete states of the whole sequence). */
int lasp_bidir_bwd(const lasp_shape *shape, const void *k, const void *v, const void *dout,
                   const float *kv, const float *dkv, void *dq, void *dk, void *dv,
                   void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LASP_H */
