/*
 * pruner.h - C boundary of the draft-then-verify schedule-exploration library for AMD gfx950.
 *
 * The library runs the data-parallel part of one exploration round of Pruner
 * (Alg. 1: S_spec <- LatentScheduleExplorer, S_measured <- PaCostModel):
 *
 *   pruner_draft_score   C_SA(sch, d) for every schedule of a population   (Alg. 2; Table 2; Sec. 4.1; Eq. 1)
 *   pruner_topk          PriorFilter / selection of the best k per subgraph (Alg. 2, PriorFilter; Alg. 1, S_measured)
 *   pruner_verify_score  statement-feature branch of the learned cost model (Sec. 4.2, "Pattern-aware Transformer")
 *
 * Conventions for every entry point
 *   - "host" pointers are read during the call only.  "device" pointers are memory of the current HIP device,
 *     allocated and owned by the caller; the library never allocates, frees or synchronises.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the null stream) and the call returns
 *     at once.  `workspace` is device scratch of at least pruner_workspace_bytes(...) bytes, 256-byte aligned,
 *     private to the call until the enqueued work has finished.
 *   - Return value: PRUNER_OK, or a negative PRUNER_E* code.  PRUNER_EINVAL, PRUNER_EWORKSPACE and PRUNER_ERANGE come
 *     from checks on the host before anything is enqueued: no output has been touched.  PRUNER_EHIP means that the HIP
 *     runtime refused a launch in the middle of a call: earlier launches of the call may already be on the stream, and
 *     the outputs are then undefined.  pruner_strerror() names a code.
 *   - What the library remembers between calls it remembers per device (compute-unit count, kernel attributes it has
 *     set, how many workgroups of a kernel a device holds), so calls may go to any device that is current when they are
 *     made.  It takes no locks: calls from several host threads at once are the caller's to serialise (the measurement
 *     hook pruner_time_dominant_draft_launch in particular is process-wide state).
 *   - Scores are higher-is-better everywhere, so one selection routine serves both stages.
 */
#ifndef PRUNER_H
#define PRUNER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PRUNER_OK 0
#define PRUNER_EINVAL (-1)      /* null / misaligned pointer, size or count out of range, unsupported descriptor */
#define PRUNER_EWORKSPACE (-2)  /* workspace missing or too small                                              */
#define PRUNER_ERANGE (-3)      /* a symbol of this subgraph could exceed the integer range the kernels use     */
#define PRUNER_EHIP (-4)        /* the HIP runtime refused a launch                                             */

#define PRUNER_MAX_SP 4     /* spatial axes   */
#define PRUNER_MAX_RD 3     /* reduction axes */
#define PRUNER_MAX_SLOTS 25 /* tile slots of a candidate: 4 per spatial axis, 2 or 3 per reduction axis */
#define PRUNER_MAX_AXES 7
#define PRUNER_MAX_DIMS 4   /* dimensions of a buffer */
#define PRUNER_MAX_TERMS 2  /* terms of one index expression */
#define PRUNER_MAX_SUBGRAPHS 4096
#define PRUNER_MAX_K 4096   /* largest k of pruner_topk */

#define PRUNER_NSYM 12      /* rows of the optional symbol dump, in this order: */
enum { PRUNER_SYM_S1, PRUNER_SYM_S2, PRUNER_SYM_S3, PRUNER_SYM_S4, PRUNER_SYM_S6, PRUNER_SYM_S8,
       PRUNER_SYM_S5_IN0, PRUNER_SYM_S7_IN0, PRUNER_SYM_S5_IN1, PRUNER_SYM_S7_IN1, PRUNER_SYM_S5_OUT, PRUNER_SYM_S7_OUT };

/* ablation switches of the draft model (Table 10: "w/o P_li,c", "w/o P_li,m") */
#define PRUNER_NO_COMPUTE_PENALTY 1 /* U_p = T_p */
#define PRUNER_NO_MEMORY_PENALTY 2  /* U_m = T_m */
/* Arithmetic of Eq. 1 (binary32 either way; the symbols are exact integers).
   Reference rounding: every ratio and every quotient of Eq. 1 is formed on its own as a correctly rounded division, in
   the order of the definitions; the score equals that binary32 evaluation bit for bit.
   Fused: the penalties of a statement group, all of them ratios, are multiplied out and divided once; the score is the
   value of Eq. 1 within 2^-20 relative, and a selection taken on it can differ from the reference's at the cut, between
   candidates whose scores lie within that distance of each other.
   Default: reference rounding for calls that run as one launch (populations below 2^20 candidates, where a call is
   bound by launch latency and the divisions cost nothing measurable; also larger ones whose layout does not allow
   8-byte loads: a segment start, the pitch or a pointer that is not a multiple of four candidates), fused for larger
   populations at the full load width (about 13 % faster there).  Either way a score is a function of its candidate
   alone: the same candidate scores the same bits in any population, launch shape or neighbourhood.  The two switches
   force one form for every size; setting both is an error. */
#define PRUNER_REFERENCE_ROUNDING 4
#define PRUNER_FUSED_ARITHMETIC 8

/* Device abstraction d (Alg. 1, Alg. 2): the constants of the "Hardware-aware Penalty" paragraph, Sec. 4.1.
   They describe the device the schedules are tuned FOR. */
typedef struct pruner_device {
    float T_p;       /* theoretical peak compute, flop/s                               */
    float T_m;       /* theoretical peak bandwidth of the lowest storage level, byte/s */
    int32_t m_l0;    /* L0 (register) allocation limit per thread, elements            */
    int32_t m_l1;    /* L1 (shared memory) allocation limit per block, bytes           */
    int32_t pu_l1;   /* L1 scheduling blocks active at once                            */
    int32_t n_l1;    /* scheduling size within a block (warp size)                     */
    int32_t pu_l2;   /* L2-level parallel units (SMs / CUs)                            */
    int32_t n_l2;    /* memory transaction length, elements of the subgraph's dtype    */
} pruner_device;

/* index of one buffer dimension = sum_t coef[t] * axis_variable[axis[t]]; axis[t] = -1 marks an unused term */
typedef struct pruner_dim {
    int32_t axis[PRUNER_MAX_TERMS];
    int32_t coef[PRUNER_MAX_TERMS];
} pruner_dim;

typedef struct pruner_buffer {
    int32_t ndim;                      /* 1..4, row-major, last dimension contiguous */
    pruner_dim dim[PRUNER_MAX_DIMS];
} pruner_buffer;

/*
 * One tiled reduction statement  O[sp] (+)= f(In_0[..], In_1[..])  - the fixed part of a schedule space
 * (what GenerateSketch would deliver, Alg. 2).  Axes: n_sp spatial, then n_rd reduction.
 * Split levels, outermost first.  Spatial (4): grid, virtual thread, thread, inner.  Reduction (2): outer
 * steps, shared-tile depth; (3): outer steps, middle, inner with shared-tile depth = middle * inner and
 * register step = inner.
 * frag = {0,0,0}, or the matrix-fragment shape (Sec. 6.4, 16x16x16): then thread-level factors count warps and
 * frag[0], frag[1], frag[2] apply to the inner tiles of spatial axes n_sp-2, n_sp-1 and the last reduction axis.
 */
typedef struct pruner_subgraph {
    int32_t n_sp, n_rd;
    int32_t extent[PRUNER_MAX_AXES];
    int32_t sp_levels, rd_levels;      /* 4, and 2 or 3 */
    int32_t dtype_bytes;
    int32_t frag[3];
    int32_t n_in;                      /* 1 or 2 input buffers */
    pruner_buffer in[2];
    pruner_buffer out;
    pruner_device hw;
} pruner_subgraph;

/* Weights of the statement-feature branch: 164 -> 256 -> 256 -> 1, ReLU after the first two layers.
   The struct lives on the host; every pointer in it is a DEVICE pointer.  Matrices are bfloat16 bit patterns,
   [out][in] row-major; biases are float. */
typedef struct pruner_mlp {
    const uint16_t* W1;  /* [256][164] */
    const float* b1;     /* [256]      */
    const uint16_t* W2;  /* [256][256] */
    const float* b2;     /* [256]      */
    const uint16_t* w3;  /* [256]      */
    float b3;
} pruner_mlp;

#define PRUNER_FEAT_DIM 164
#define PRUNER_MAX_STMT 8
#define PRUNER_HIDDEN 256
#define PRUNER_FLOW_DIM 23   /* temporal dataflow features of one data-movement block (Sec. 4.2) */
#define PRUNER_MAX_BLOCKS 8  /* blocks per candidate */
#define PRUNER_EMBED 64      /* width of the dataflow branch in this library's model */

/* Weights of the whole Pattern-aware Transformer (pruner_pacm_score).  The struct lives on the host; every pointer in
   it is a DEVICE pointer.  Matrices are bfloat16 bit patterns, [out][in] row-major; biases are float. */
typedef struct pruner_pacm {
    const uint16_t* W1;  /* [256][164]  statement branch */
    const float* b1;     /* [256]       */
    const uint16_t* W2;  /* [256][256]  */
    const float* b2;     /* [256]       */
    const uint16_t* We;  /* [64][23]    dataflow branch: embedding */
    const float* be;     /* [64]        */
    const uint16_t* Wq;  /* [64][64]    attention (no biases) */
    const uint16_t* Wk;  /* [64][64]    */
    const uint16_t* Wv;  /* [64][64]    */
    const uint16_t* Wo;  /* [64][64]    */
    const uint16_t* Wh;  /* [256][320]  head: columns 0..255 take the statement branch, 256..319 the dataflow branch */
    const float* bh;     /* [256]       */
    const uint16_t* wo;  /* [256]       */
    float bo;
} pruner_pacm;

/*
 * Draft model: score[c] = -L_total(c) for every candidate c (Alg. 2, C_SA; Eq. 1).
 *
 *   sg        host   [n_sg]      subgraph descriptors
 *   seg_off   host   [n_sg+1]    candidates of subgraph s are [seg_off[s], seg_off[s+1]); seg_off[0] = 0, non-decreasing
 *   tiles     device uint16      tiles[slot * tiles_pitch + c]: tile factors, structure of arrays; slot = axis-major,
 *                                then level, outermost first.  A subgraph reads its first n_sp*4 + n_rd*rd_levels slots.
 *                                Every factor must be >= 1 and the factors of an axis must multiply to its extent
 *                                (not checked; otherwise that candidate's score is meaningless, nothing else is harmed).
 *   tiles_pitch                  elements between slots, >= seg_off[n_sg]
 *   flags                        0, or PRUNER_NO_* switches and at most one of the two arithmetic switches
 *   score     device float [n]   out
 *   symbols   device int64       out or NULL: symbols[r * n + c], rows PRUNER_SYM_*
 *
 * The symbols are exact integers.  Penalties, utilisation and latency are evaluated in binary32, in the form the flags
 * select (see PRUNER_REFERENCE_ROUNDING above; the order of operations is in the kernel source).
 * Unroll / vectorise annotations of a candidate do not enter the draft model and are not an argument: Table 2's
 * symbols do not read them.  A caller keeps them beside the tile factors and carries them to the verify stage.
 * workspace: pruner_workspace_bytes(PRUNER_WS_DRAFT, n, n_sg, 0).
 */
int pruner_draft_score(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off,
                       const uint16_t* tiles, int64_t tiles_pitch, int32_t flags,
                       float* score, int64_t* symbols,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement hook, not part of the method: from now on every call that scores a population (pruner_draft_score,
 * pruner_prior_filter, pruner_lse) records `start_event` right before and `stop_event` right after the one draft
 * kernel launch of the call that covers the most candidates (a call launches one kernel per loop-nest class), on the
 * call's stream, and stores that launch's algorithmic bytes (candidates x (2 x tile slots + 4)) in
 * *algorithmic_bytes (host, may be NULL).  Both events NULL switches the hook off.  The events are the caller's
 * (hipEvent_t); process-wide state, not thread-safe: for benchmarks.
 * Errors: PRUNER_EINVAL if exactly one event is NULL.
 */
int pruner_time_dominant_draft_launch(void* start_event, void* stop_event, int64_t* algorithmic_bytes);

/*
 * Selection: for every segment the k best entries, best first, ordered by (score descending, index ascending).
 *
 *   score    device float [n]       must not hold NaN; -0.0 and +0.0 compare equal; infinities are ordinary values
 *   seg_off  host   [n_sg+1]        as above; every segment must hold at least k entries
 *   k                               1..PRUNER_MAX_K
 *   idx_out  device int32 [n_sg*k]  idx_out[s*k + r] = global index of rank r of segment s
 *   val_out  device float [n_sg*k]  the matching scores, or NULL
 * workspace: pruner_workspace_bytes(PRUNER_WS_TOPK, n, n_sg, k).
 */
int pruner_topk(const float* score, const int64_t* seg_off, int32_t n_sg, int32_t k,
                int32_t* idx_out, float* val_out,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * PriorFilter of Alg. 2 in one call: the draft score C_SA of every candidate (as pruner_draft_score, without the
 * symbol dump), then the k best candidates of every subgraph (as pruner_topk on those scores).  Same arguments,
 * same results bit for bit, as the two calls in sequence; the saving is that the selection's first counting
 * pass rides along in the draft kernel when the population is large.
 *
 *   score         device float [n]         out: all draft scores (also the selection's input)
 *   idx_out       device int32 [n_sg*k]    out
 *   val_out       device float [n_sg*k]    out, or NULL
 *   scored_event  hipEvent_t or NULL       recorded on `stream` after the draft-score launches and before the
 *                                          selection launches (lets a caller time the two stages apart)
 * workspace: pruner_workspace_bytes(PRUNER_WS_PRIOR_FILTER, n, n_sg, k).
 * Errors: those of pruner_draft_score and pruner_topk (every segment needs at least k candidates).
 */
int pruner_prior_filter(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off,
                        const uint16_t* tiles, int64_t tiles_pitch, int32_t flags, int32_t k,
                        float* score, int32_t* idx_out, float* val_out,
                        void* workspace, size_t workspace_bytes, void* stream, void* scored_event);

/*
 * Latent Schedule Explorer, Alg. 2, with the population resident on the device:
 *     repeat n_steps times:  costs = C_SA(S_x);  S_spec = PriorFilter(S_x U S_spec, costs);  S_x = SchMutation(S_x, costs)
 * C_SA and the k best of S_x are computed as by pruner_prior_filter (same flags).
 * PriorFilter keeps the k best of the union of SETS: a schedule counts once (identity: equal score and equal 64-bit
 * hash of its tile factors).  The union is ordered by score descending, then hash ascending, then age (S_spec's
 * entries before S_x's, then position); a copy of its predecessor is dropped; the first k remain.
 * SchMutation (the paper names a genetic algorithm over tiling factors guided by the draft fitness; the operator is
 * this library's): child j copies member floor(low32(draw 1) * spec_count / 2^32) of its subgraph's S_spec and, with probability
 * mutate_q16 / 65536, moves one prime factor of one tile factor to another level of the same axis (fragment multiples
 * are kept; a move that would break one leaves the child a plain copy).  Random numbers: draw c is the c-th output of
 * SplitMix64 started from `seed`; child j in step t uses draws (t << 41) + 2 j + 1 and + 2.
 *
 *   tiles       device uint16 [tile_rows][tiles_pitch]  in: the initial S_x; out: S_x after the last mutation
 *   score       device float [n]                        out: C_SA of the last population that was scored
 *   spec_tiles  device uint16 [tile_rows][n_sg*k]       out: S_spec, best first; rows a subgraph does not own and
 *   spec_score  device float [n_sg*k]                        entries past spec_count hold 0 / -infinity
 *   spec_count  device int32 [n_sg]                     out: members of S_spec per subgraph (<= k)
 * workspace: pruner_workspace_bytes(PRUNER_WS_LSE, n, n_sg, k).
 * Errors: those of pruner_prior_filter; PRUNER_EINVAL also for n_steps < 1, mutate_q16 > 65536, tile_rows below a
 * subgraph's slot count or above PRUNER_MAX_SLOTS.
 */
int pruner_lse(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off,
               uint16_t* tiles, int64_t tiles_pitch, int32_t tile_rows, int32_t flags,
               int32_t k, int32_t n_steps, uint64_t seed, uint32_t mutate_q16,
               float* score, uint16_t* spec_tiles, float* spec_score, int32_t* spec_count,
               void* workspace, size_t workspace_bytes, void* stream);

/*
 * RandomInitSch (Alg. 1: S_draft = S_spec U RandomInitSch(p0); Alg. 2: the initial S_x): every candidate of every
 * segment becomes a schedule drawn uniformly from its subgraph's schedule space.  (The paper says that schedules are
 * sampled at random and no more; the numbering below is this library's.)
 * A schedule is one ordered factorisation of every axis extent into the axis's levels, the axes independent; in
 * fragment mode the innermost factor of spatial axes n_sp-2, n_sp-1 and of the last reduction axis is a multiple of
 * frag[0], frag[1], frag[2]: extent / frag is factorised and the innermost factor multiplied by frag.
 * The ordered L-factorisations of b = p1^e1 p2^e2 ... (primes ascending) are numbered R = r_1 + C_1 (r_2 + C_2 (...)):
 * r_i is the lexicographic rank of the weak composition of e_i into L parts (part l = exponent of p_i in the factor of
 * level l, outermost first), C_i = binom(e_i + L - 1, L - 1).  Candidate c (global index), axis a (spatial axes
 * first) takes R = floor(u * count / 2^64), u = draw number 8 c + a + 1 of SplitMix64 started from `seed`.
 * The result depends on (seed, c, subgraph) only, not on how a population is cut into calls or segments.
 *
 *   sg, seg_off  host        as for pruner_draft_score (only n_sp, n_rd, extent, rd_levels, frag are read)
 *   tiles        device uint16 [tile_rows][tiles_pitch]  out; rows a subgraph does not own are cleared
 *   tile_rows                >= the largest slot count of the call, <= PRUNER_MAX_SLOTS
 * workspace: pruner_random_init_workspace_bytes(sg, n_sg) (the tables R -> factors of the call's axis spaces); 0 from
 * that function means the descriptors are invalid.
 * Errors: PRUNER_EINVAL for bad pointers, sizes or descriptors (an extent outside 1..65535 or not a multiple of its
 * fragment size); PRUNER_ERANGE if the tables would exceed 2^31 rows; PRUNER_EWORKSPACE.
 */
size_t pruner_random_init_workspace_bytes(const pruner_subgraph* sg, int32_t n_sg);
int pruner_random_init(const pruner_subgraph* sg, int32_t n_sg, const int64_t* seg_off,
                       uint16_t* tiles, int64_t tiles_pitch, int32_t tile_rows, uint64_t seed,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * The whole Pattern-aware Transformer (Sec. 4.2): statement features through linear layers and a sum over statements,
 * temporal dataflow features through self-attention, concatenation, linear head.  The paper's figure with the model's
 * dimensions is not reproduced in its text; this library's model:
 *   statement s < n_stmt[c]:  h1 = relu(W1 x_s + b1);  h2 = relu(W2 h1 + b2);        v_s = sum_s h2        (256)
 *   block i < n_blk[c]:       e_i = relu(We d_i + be);  q_i, k_i, v_i = Wq e_i, Wk e_i, Wv e_i
 *                             a_ij = softmax_j(q_i . k_j / 8),  o_i = sum_j a_ij v_j
 *                             z_i = e_i + Wo o_i;                                   v_d = sum_i z_i       (64)
 *   head:                     g = relu(Wh [v_s ; v_d] + bh);  y[c] = wo . g + bo
 * Every operand of a matrix product is rounded to bfloat16 (inputs, e, q, k, v, o, h1, h2, the pooled vectors), products
 * are accumulated in binary32, the softmax is binary32.  A candidate without blocks has v_d = 0.
 *
 *   feat    device float [n_d][8][164]   statement features; rows s >= n_stmt[c] are ignored whatever they hold
 *   n_stmt  device int32 [n_d]           0..8 (values outside are clamped)
 *   flow    device float [n_d][8][23]    dataflow features; rows i >= n_blk[c] are ignored whatever they hold
 *   n_blk   device int32 [n_d]           0..8 (values outside are clamped)
 *   y       device float [n_d]           out
 * workspace: pruner_workspace_bytes(PRUNER_WS_PACM, n_d, 0, 0) (the pooled vectors of the two branches).
 * Errors: PRUNER_EINVAL (null or misaligned pointers: feat, W2, Wh 16 bytes, W1 8 bytes), PRUNER_EWORKSPACE.
 */
int pruner_pacm_score(const float* feat, const int32_t* n_stmt, const float* flow, const int32_t* n_blk, int64_t n_d,
                      const pruner_pacm* w, float* y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Momentum online Adaptation (Sec. 4.3; Update_MoA of Alg. 1; the paper's m is 0.99): the Siamese model's weights
 * follow the target model's after a round of fine-tuning,  phi_s <- m phi_s + (1 - m) phi_t.
 * (The formula sits in a figure the text does not reproduce; this is the momentum-contrast form, which equals
 * phi_s - (1 - m) lr sum Delta_t for phi_t = phi_s - lr sum Delta_t.)  binary32, each operation rounded on its own:
 * c = 1 - m;  phi_s = (m * phi_s) + (c * phi_t).
 *
 *   phi_s       device float [n]     in/out: the Siamese model's weights, any flat order
 *   phi_t       device float [n]     the target model's weights in the same order
 *   m                                0 <= m <= 1
 *   phi_s_bf16  device uint16 [n]    out or NULL: the new phi_s as bfloat16 (nearest, ties to even), e.g. the W1 / W2 /
 *                                    w3 of a pruner_mlp
 * No workspace.  Errors: PRUNER_EINVAL (null or misaligned pointers, n < 0, m outside [0, 1] or NaN).
 */
int pruner_moa_update(float* phi_s, const float* phi_t, int64_t n, float m, uint16_t* phi_s_bf16, void* stream);

/*
 * Verify model: vscore[c] = sum over s < n_stmt[c] of  w3 . relu(W2 relu(W1 x_cs + b1) + b2) + b3
 * (statement features through linear layers, then summation over statements, Sec. 4.2).
 *
 *   feat     device float [n_d][8][164]   per-statement features; rows s >= n_stmt[c] are ignored whatever they hold
 *   n_stmt   device int32 [n_d]           valid rows, 0..8
 *   w        host struct of device pointers
 *   vscore   device float [n_d]           out
 * Inputs and hidden activations are rounded to bfloat16 (nearest even); products accumulate in binary32 on the
 * matrix cores.
 * workspace: pruner_workspace_bytes(PRUNER_WS_VERIFY, n_d, 0, 0) (256 bytes, not used at present: the stage keeps its
 * row numbering in on-chip memory).
 */
int pruner_verify_score(const float* feat, const int32_t* n_stmt, int64_t n_d, const pruner_mlp* w,
                        float* vscore, void* workspace, size_t workspace_bytes, void* stream);

/*
 * pruner_topk for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same results bit for bit as pruner_topk; the scratch
 * lives in an 8 MiB array inside the library's device image (one per device, held until the process ends), which
 * limits the call to PRUNER_STATIC_MAX_SEGMENTS segments (any n up to 2^31 - 1, any k up to PRUNER_MAX_K).  The call
 * allocates nothing, on the device or on the host.  Every call on a device shares that device's array: calls that overlap on one device (two
 * streams, two threads) race; calls on one stream are ordered and safe.
 * Errors: those of pruner_topk; PRUNER_EINVAL for n_sg above the limit; PRUNER_EHIP if the array's address cannot be
 * looked up on the current device.
 */
#define PRUNER_STATIC_MAX_SEGMENTS 16
int pruner_topk_static(const float* score, const int64_t* seg_off, int32_t n_sg, int32_t k,
                       int32_t* idx_out, float* val_out, void* stream);

#define PRUNER_WS_DRAFT 0
#define PRUNER_WS_TOPK 1
#define PRUNER_WS_VERIFY 2
#define PRUNER_WS_PRIOR_FILTER 3
#define PRUNER_WS_LSE 4
#define PRUNER_WS_PACM 5          /* n = candidates of the drafted set */

/* Bytes of workspace entry point `which` needs for n items in n_sg segments with selection size k (0 if unused). */
size_t pruner_workspace_bytes(int32_t which, int64_t n, int32_t n_sg, int32_t k);

/* Static, read-only description of a return code. */
const char* pruner_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* PRUNER_H */
