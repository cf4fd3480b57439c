/*
 * CPU oracle for the draft-then-verify exploration path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar implementation of what the path computes, written from
 * the paper, one step per statement, with no blocking, fusion or reordering:
 *
 *   orc_symbols      hardware-aware symbols S1..S8          (Table 2; Sec. 4.1 "Hardware-aware Symbols")
 *   orc_analyze_*    penalties, utilisation, latency        (Sec. 4.1 "Hardware-aware Penalty"; Eq. 1)
 *   orc_draft_score  C_SA over a population                 (Alg. 2, function C_SA and the loop over S_x)
 *   orc_topk         PriorFilter / final selection          (Alg. 2 PriorFilter; Alg. 1 S_measured)
 *   orc_verify       statement-feature branch of the model  (Sec. 4.2 "Pattern-aware Transformer": linear
 *                                                            layers on statement features, then summation)
 *   orc_lse          the explorer loop                      (Alg. 2: C_SA, PriorFilter over the union, SchMutation)
 *   orc_random_init  uniform schedules of a subgraph        (Alg. 1 RandomInitSch; Alg. 2's initial S_x)
 *   orc_pacm         the whole cost model                   (Sec. 4.2: statement branch, self-attention over
 *                                                            dataflow blocks, concatenation, linear head)
 *   orc_moa_update   momentum update of the Siamese weights (Sec. 4.3)
 * (the last four follow readings of passages in which the paper gives no operator, dimensions or formula; each
 * states its reading where it is defined, and the tests pin each from outside this file: traces in plain integers
 * from the published generator, closed forms, brute-force enumeration, hand-sized cases)
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call this
 * file.  It shares no code, header, table or constant with the HIP library and
 * is never a fallback for it.
 *
 * Precision.  The paper fixes none.  Every floating-point quantity is computed
 * twice from the same integer symbols: in binary64 (the reference value), and
 * in binary32 with every operation rounded separately in the order written
 * below (the precision in which the top-k decision is taken, so that selection
 * can be compared index by index).  Build with -ffp-contract=off.
 *
 * Readings of the paper (its Figure 3, which showed the symbol extraction for
 * a GEMM, is not available; none of these is pinned by a value the paper
 * prints - "parity unpinned" for them; they are pinned by hand-computed
 * examples, closed forms and brute force in the tests):
 *   - split levels of a spatial axis, outermost first: grid (G), virtual
 *     thread (V), thread (T), inner (I); of a reduction axis: outer steps (O)
 *     then shared-tile depth (D = f1, q = 1) for 2 levels, or O, D = f1*f2,
 *     q = f2 for 3 levels.  Block tile B = V*T*I, thread tile R = V*I.
 *   - statements of a subgraph: one load per input buffer, the compute
 *     statement, one store.  S1,S2,S3,S4,S6 describe the whole program;
 *     S5,S7 belong to a memory statement, S8 to the compute statement.
 *   - alpha_l1 multiplies U_p; all three memory penalties multiply U_m.
 *   - footprints are affine tile extents, image borders ignored.
 *   - fragment (matrix-core) mode: thread-level factors count warps; see
 *     orc_symbols and orc_analyze_*.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAX_AXES 7
#define ORC_MAX_DIMS 4
#define ORC_MAX_TERMS 2
#define ORC_NSYM 12

/* ablation switches of Table 10 */
#define ORC_NO_COMPUTE_PENALTY 1 /* U_p = T_p            */
#define ORC_NO_MEMORY_PENALTY 2  /* U_m = T_m            */

typedef struct {
    float T_p, T_m;
    int32_t m_l0, m_l1, pu_l1, n_l1, pu_l2, n_l2;
} orc_device;

typedef struct {
    int32_t axis[ORC_MAX_TERMS]; /* -1 = unused term */
    int32_t coef[ORC_MAX_TERMS];
} orc_dim;

typedef struct {
    int32_t ndim;
    orc_dim dim[ORC_MAX_DIMS];
} orc_buffer;

typedef struct {
    int32_t n_sp, n_rd;
    int32_t extent[ORC_MAX_AXES];
    int32_t sp_levels, rd_levels;
    int32_t dtype_bytes;
    int32_t frag[3];
    int32_t n_in;
    orc_buffer in[2];
    orc_buffer out;
    orc_device hw;
} orc_subgraph;

/* symbol slots of the 12-entry vector */
enum { SYM_S1, SYM_S2, SYM_S3, SYM_S4, SYM_S6, SYM_S8, SYM_S5_IN0, SYM_S7_IN0, SYM_S5_IN1, SYM_S7_IN1, SYM_S5_OUT, SYM_S7_OUT };

static int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

/* extent of one buffer dimension over a tile with per-axis extents e[]: 1 + sum coef*(e-1) */
static int64_t dim_extent(const orc_dim* d, const int64_t* e)
{
    int64_t ext = 1;
    for (int t = 0; t < ORC_MAX_TERMS; ++t)
        if (d->axis[t] >= 0) ext += (int64_t)d->coef[t] * (e[d->axis[t]] - 1);
    return ext;
}

static int64_t footprint(const orc_buffer* b, const int64_t* e)
{
    int64_t fp = 1;
    for (int d = 0; d < b->ndim; ++d) fp *= dim_extent(&b->dim[d], e);
    return fp;
}

static int in_fragment_mode(const orc_subgraph* sg) { return sg->frag[0] > 0; }

static int check_subgraph(const orc_subgraph* sg)
{
    if (sg->n_sp < 1 || sg->n_sp > 4 || sg->n_rd < 0 || sg->n_rd > 3) return -1;
    if (sg->sp_levels != 4 || (sg->rd_levels != 2 && sg->rd_levels != 3)) return -1;
    if (sg->n_in < 1 || sg->n_in > 2 || sg->dtype_bytes < 1) return -1;
    if (in_fragment_mode(sg) && (sg->n_sp < 2 || sg->n_rd < 1 || sg->frag[1] <= 0 || sg->frag[2] <= 0)) return -1;
    const orc_device* d = &sg->hw;
    if (!(d->T_p > 0) || !(d->T_m > 0) || d->m_l0 < 1 || d->m_l1 < 1 || d->pu_l1 < 1 || d->n_l1 < 1 || d->pu_l2 < 1 || d->n_l2 < 1) return -1;
    return 0;
}

/*
 * Hardware-aware symbols of one candidate (Table 2).
 * f[slot * stride]: tile factors, axis-major, outermost level first.
 * Returns 0, or -2 if a factor is 0 or an axis's factors do not multiply to its extent.
 */
int orc_symbols(const orc_subgraph* sg, const uint16_t* f, int64_t stride, int64_t* sym)
{
    if (check_subgraph(sg)) return -1;
    const int n_axes = sg->n_sp + sg->n_rd;
    int64_t G[4], V[4], T[4], I[4]; /* spatial levels                              */
    int64_t O[3], D[3], q[3];       /* reduction: outer steps, shared depth, reg step */
    int64_t e_blk[ORC_MAX_AXES], e_reg[ORC_MAX_AXES];

    int slot = 0;
    for (int a = 0; a < sg->n_sp; ++a, slot += 4) {
        G[a] = f[(slot + 0) * stride];
        V[a] = f[(slot + 1) * stride];
        T[a] = f[(slot + 2) * stride];
        I[a] = f[(slot + 3) * stride];
        if (G[a] * V[a] * T[a] * I[a] != sg->extent[a] || sg->extent[a] == 0) return -2;
        e_blk[a] = V[a] * T[a] * I[a]; /* block tile  B_a */
        e_reg[a] = V[a] * I[a];        /* thread tile R_a */
    }
    for (int r = 0; r < sg->n_rd; ++r, slot += sg->rd_levels) {
        const int a = sg->n_sp + r;
        O[r] = f[slot * stride];
        if (sg->rd_levels == 2) {
            D[r] = f[(slot + 1) * stride];
            q[r] = 1;
        } else {
            q[r] = f[(slot + 2) * stride];
            D[r] = (int64_t)f[(slot + 1) * stride] * q[r];
        }
        if (O[r] * D[r] != sg->extent[a] || sg->extent[a] == 0) return -2;
        e_blk[a] = D[r];
        e_reg[a] = q[r];
    }

    int64_t prod_R = 1, prod_T = 1, prod_G = 1, prod_q = 1, prod_O = 1, prod_sp = 1, prod_all = 1;
    for (int a = 0; a < sg->n_sp; ++a) {
        prod_R *= e_reg[a];
        prod_T *= T[a];
        prod_G *= G[a];
        prod_sp *= sg->extent[a];
    }
    for (int r = 0; r < sg->n_rd; ++r) {
        prod_q *= q[r];
        prod_O *= O[r];
    }
    for (int a = 0; a < n_axes; ++a) prod_all *= sg->extent[a];

    /* S1 L0MemAlloc: accumulators + operand registers of one register-tile step, elements */
    int64_t S1 = prod_R;
    for (int b = 0; b < sg->n_in; ++b) S1 += footprint(&sg->in[b], e_reg);
    /* S2 L0CompCount: flops of one register-tile step */
    int64_t S2 = 2 * prod_R * prod_q;
    /* S3 L1MemAlloc: shared bytes per block */
    int64_t S3 = 0;
    for (int b = 0; b < sg->n_in; ++b) S3 += footprint(&sg->in[b], e_blk);
    S3 *= sg->dtype_bytes;
    /* S4 L1ParaInfo: threads per block */
    int64_t S4 = prod_T;
    /* S6 L2ParaInfo: blocks in the grid */
    int64_t S6 = prod_G;
    /* S8 L2CompCount: flops of the statement, independent of the tiling */
    int64_t S8 = 2 * prod_all;

    if (in_fragment_mode(sg)) {
        /* thread-level factors count warps: a block has n_l1 * prod(T) lanes and the
           register tile of a warp is shared out over its n_l1 lanes */
        S4 = (int64_t)sg->hw.n_l1 * prod_T;
        S1 = cdiv(S1, sg->hw.n_l1);
    }

    memset(sym, 0, ORC_NSYM * sizeof(int64_t));
    sym[SYM_S1] = S1;
    sym[SYM_S2] = S2;
    sym[SYM_S3] = S3;
    sym[SYM_S4] = S4;
    sym[SYM_S6] = S6;
    sym[SYM_S8] = S8;
    /* S5 L2MemFootprint of a load: every block reads its tile once per outer reduction step;
       S7 L2TransDim: contiguous run (innermost dimension) of that tile, elements */
    for (int b = 0; b < sg->n_in; ++b) {
        const orc_buffer* X = &sg->in[b];
        sym[SYM_S5_IN0 + 2 * b] = (int64_t)sg->dtype_bytes * S6 * prod_O * footprint(X, e_blk);
        sym[SYM_S7_IN0 + 2 * b] = dim_extent(&X->dim[X->ndim - 1], e_blk);
    }
    /* store: the output is written once */
    sym[SYM_S5_OUT] = (int64_t)sg->dtype_bytes * prod_sp;
    sym[SYM_S7_OUT] = dim_extent(&sg->out.dim[sg->out.ndim - 1], e_blk);
    return 0;
}

/* fragment-utilisation numerator / denominator: inner tile over the tile rounded up to whole fragments */
static void fragment_ratio(const orc_subgraph* sg, const uint16_t* f, int64_t stride, int64_t* num, int64_t* den)
{
    const int ai = sg->n_sp - 2, aj = sg->n_sp - 1, rk = sg->n_rd - 1;
    int64_t Ii = f[(ai * 4 + 3) * stride];
    int64_t Ij = f[(aj * 4 + 3) * stride];
    int64_t qk = sg->rd_levels == 3 ? f[(sg->n_sp * 4 + rk * 3 + 2) * stride] : 1;
    *num = Ii * Ij * qk;
    *den = cdiv(Ii, sg->frag[0]) * sg->frag[0] * cdiv(Ij, sg->frag[1]) * sg->frag[1] * cdiv(qk, sg->frag[2]) * sg->frag[2];
}

/* slots of the term vector filled by orc_analyze_f64 / orc_analyze_f32 */
enum { TRM_P0M, TRM_P0C, TRM_P1M, TRM_P1C, TRM_ALPHA, TRM_P2C, TRM_PTC, TRM_UP, TRM_LC,
       TRM_P2M_IN0, TRM_UM_IN0, TRM_LM_IN0, TRM_P2M_IN1, TRM_UM_IN1, TRM_LM_IN1, TRM_P2M_OUT, TRM_UM_OUT, TRM_LM_OUT, TRM_LTOTAL, ORC_NTERM };

/*
 * Penalties (Sec. 4.1 "Hardware-aware Penalty"), utilisation and latency (Eq. 1), binary64.
 * frag_num/frag_den: fragment ratio (1/1 outside fragment mode).  Returns L_total.
 */
double orc_analyze_f64(const orc_subgraph* sg, const int64_t* sym, int64_t frag_num, int64_t frag_den, int32_t flags, double* term)
{
    const orc_device* d = &sg->hw;
    double t[ORC_NTERM];
    memset(t, 0, sizeof t);
    const int64_t S1 = sym[SYM_S1], S2 = sym[SYM_S2], S3 = sym[SYM_S3], S4 = sym[SYM_S4], S6 = sym[SYM_S6], S8 = sym[SYM_S8];

    t[TRM_P0M] = fmin((double)d->m_l0 / (double)S1, 1.0);
    t[TRM_P0C] = 1.0 + (double)S2 / (double)S1;
    t[TRM_P1M] = fmin((double)d->m_l1 / (double)S3, 1.0);
    const int64_t sch = cdiv(S4, d->n_l1);
    t[TRM_P1C] = (double)sch / (double)(cdiv(sch, d->pu_l1) * d->pu_l1);
    t[TRM_ALPHA] = (double)S4 / (double)(sch * d->n_l1);
    t[TRM_P2C] = (double)S6 / (double)(cdiv(S6, d->pu_l2) * d->pu_l2);
    t[TRM_PTC] = (double)frag_num / (double)frag_den;

    double Up = (double)d->T_p;
    if (!(flags & ORC_NO_COMPUTE_PENALTY)) {
        Up = (((Up * t[TRM_P0C]) * t[TRM_P1C]) * t[TRM_ALPHA]) * t[TRM_P2C];
        if (in_fragment_mode(sg)) Up = Up * t[TRM_PTC];
    }
    t[TRM_UP] = Up;
    t[TRM_LC] = (double)S8 / Up;
    double L = t[TRM_LC];

    for (int s = 0; s < 3; ++s) { /* memory statements: In_0, In_1, store */
        if (s < 2 && s >= sg->n_in) continue;
        const int64_t S5 = sym[SYM_S5_IN0 + 2 * s], S7 = sym[SYM_S7_IN0 + 2 * s];
        const double P2m = (double)S7 / (double)(cdiv(S7, d->n_l2) * d->n_l2);
        double Um = (double)d->T_m;
        if (!(flags & ORC_NO_MEMORY_PENALTY)) Um = ((Um * t[TRM_P0M]) * t[TRM_P1M]) * P2m;
        const double Lm = (double)S5 / Um;
        t[TRM_P2M_IN0 + 3 * s] = P2m;
        t[TRM_UM_IN0 + 3 * s] = Um;
        t[TRM_LM_IN0 + 3 * s] = Lm;
        L = L + Lm;
    }
    t[TRM_LTOTAL] = L;
    if (term) memcpy(term, t, sizeof t);
    return L;
}

/* The same steps, every operation rounded to binary32 (conversions round to nearest even). */
float orc_analyze_f32(const orc_subgraph* sg, const int64_t* sym, int64_t frag_num, int64_t frag_den, int32_t flags, float* term)
{
    const orc_device* d = &sg->hw;
    float t[ORC_NTERM];
    memset(t, 0, sizeof t);
    const int64_t S1 = sym[SYM_S1], S2 = sym[SYM_S2], S3 = sym[SYM_S3], S4 = sym[SYM_S4], S6 = sym[SYM_S6], S8 = sym[SYM_S8];

    t[TRM_P0M] = fminf((float)d->m_l0 / (float)S1, 1.0f);
    t[TRM_P0C] = 1.0f + (float)S2 / (float)S1;
    t[TRM_P1M] = fminf((float)d->m_l1 / (float)S3, 1.0f);
    const int64_t sch = cdiv(S4, d->n_l1);
    t[TRM_P1C] = (float)sch / (float)(cdiv(sch, d->pu_l1) * d->pu_l1);
    t[TRM_ALPHA] = (float)S4 / (float)(sch * d->n_l1);
    t[TRM_P2C] = (float)S6 / (float)(cdiv(S6, d->pu_l2) * d->pu_l2);
    t[TRM_PTC] = (float)frag_num / (float)frag_den;

    float Up = d->T_p;
    if (!(flags & ORC_NO_COMPUTE_PENALTY)) {
        Up = (((Up * t[TRM_P0C]) * t[TRM_P1C]) * t[TRM_ALPHA]) * t[TRM_P2C];
        if (in_fragment_mode(sg)) Up = Up * t[TRM_PTC];
    }
    t[TRM_UP] = Up;
    t[TRM_LC] = (float)S8 / Up;
    float L = t[TRM_LC];

    for (int s = 0; s < 3; ++s) {
        if (s < 2 && s >= sg->n_in) continue;
        const int64_t S5 = sym[SYM_S5_IN0 + 2 * s], S7 = sym[SYM_S7_IN0 + 2 * s];
        const float P2m = (float)S7 / (float)(cdiv(S7, d->n_l2) * d->n_l2);
        float Um = d->T_m;
        if (!(flags & ORC_NO_MEMORY_PENALTY)) Um = ((Um * t[TRM_P0M]) * t[TRM_P1M]) * P2m;
        const float Lm = (float)S5 / Um;
        t[TRM_P2M_IN0 + 3 * s] = P2m;
        t[TRM_UM_IN0 + 3 * s] = Um;
        t[TRM_LM_IN0 + 3 * s] = Lm;
        L = L + Lm;
    }
    t[TRM_LTOTAL] = L;
    if (term) memcpy(term, t, sizeof t);
    return L;
}

/* L_total of one candidate with all intermediate terms, for the tests that pin single formulas. */
int orc_analyze_candidate(const orc_subgraph* sg, const uint16_t* f, int64_t stride, int32_t flags,
                          int64_t* sym, double* term64, float* term32)
{
    int64_t s[ORC_NSYM];
    int rc = orc_symbols(sg, f, stride, s);
    if (rc) return rc;
    int64_t num = 1, den = 1;
    if (in_fragment_mode(sg)) fragment_ratio(sg, f, stride, &num, &den);
    if (sym) memcpy(sym, s, sizeof s);
    orc_analyze_f64(sg, s, num, den, flags, term64);
    orc_analyze_f32(sg, s, num, den, flags, term32);
    return 0;
}

/*
 * C_SA over a population (Alg. 2).  Candidates of subgraph s are [seg_off[s], seg_off[s+1]);
 * tiles[slot * pitch + c].  The draft score is the fitness F = -L_total (higher is better).
 * score32 / score64 / feat ([ORC_NSYM][n], row stride n) may each be NULL.
 */
int orc_draft_score(const orc_subgraph* sg, int32_t n_sg, const int64_t* seg_off, const uint16_t* tiles, int64_t pitch,
                    int32_t flags, float* score32, double* score64, int64_t* feat)
{
    const int64_t n = seg_off[n_sg];
    for (int32_t s = 0; s < n_sg; ++s) {
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            int64_t sym[ORC_NSYM];
            int rc = orc_symbols(&sg[s], tiles + c, pitch, sym);
            if (rc) return rc;
            int64_t num = 1, den = 1;
            if (in_fragment_mode(&sg[s])) fragment_ratio(&sg[s], tiles + c, pitch, &num, &den);
            if (feat)
                for (int k = 0; k < ORC_NSYM; ++k) feat[k * n + c] = sym[k];
            if (score64) {
                double L = orc_analyze_f64(&sg[s], sym, num, den, flags, NULL);
                if (isnan(L)) return -3;
                score64[c] = -L;
            }
            if (score32) {
                float L = orc_analyze_f32(&sg[s], sym, num, den, flags, NULL);
                if (isnan(L)) return -3;
                score32[c] = -L;
            }
        }
    }
    return 0;
}

/* ---- selection ------------------------------------------------------------------------ */

typedef struct {
    float score;
    int64_t idx;
} orc_pair;

/* best first: higher score, then lower index.  -0.0 and +0.0 compare equal. */
static int by_score_then_index(const void* pa, const void* pb)
{
    const orc_pair* a = (const orc_pair*)pa;
    const orc_pair* b = (const orc_pair*)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

/*
 * Per segment, the k best entries in order (rank 0 best): a full sort of the segment by
 * (score descending, global index ascending), cut at k.  idx_out[s*k + r], val_out[s*k + r].
 * Errors: -1 bad argument or k larger than a segment, -3 NaN score.
 */
int orc_topk(const float* score, const int64_t* seg_off, int32_t n_sg, int32_t k, int32_t* idx_out, float* val_out)
{
    if (n_sg <= 0 || k <= 0) return -1;
    for (int32_t s = 0; s < n_sg; ++s)
        if (seg_off[s + 1] - seg_off[s] < k) return -1;
    for (int32_t s = 0; s < n_sg; ++s) {
        const int64_t lo = seg_off[s], len = seg_off[s + 1] - lo;
        orc_pair* p = (orc_pair*)malloc((size_t)len * sizeof(orc_pair));
        if (!p) return -4;
        for (int64_t i = 0; i < len; ++i) {
            if (isnan(score[lo + i])) {
                free(p);
                return -3;
            }
            p[i].score = score[lo + i];
            p[i].idx = lo + i;
        }
        qsort(p, (size_t)len, sizeof(orc_pair), by_score_then_index);
        for (int32_t r = 0; r < k; ++r) {
            idx_out[(int64_t)s * k + r] = (int32_t)p[r].idx;
            if (val_out) val_out[(int64_t)s * k + r] = p[r].score;
        }
        free(p);
    }
    return 0;
}

/* ---- learned cost model, statement-feature branch ---------------------------------------- */

/* binary32 -> nearest bfloat16 (ties to even), returned widened back to binary32 */
float orc_bf16_round(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return x; /* inf / nan unchanged */
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&x, &u, 4);
    return x;
}

static float bf16_bits_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float x;
    memcpy(&x, &u, 4);
    return x;
}

/*
 * vscore[c] = sum over valid statements s < n_stmt[c] of
 *     y_s = w3 . relu(W2 relu(W1 x_s + b1) + b2) + b3
 * feat [n_d][max_stmt][feat_dim] binary32; W1 [hidden][feat_dim], W2 [hidden][hidden], w3 [hidden] bfloat16 bits;
 * b1, b2 [hidden] binary32.
 * vscore32: inputs and hidden activations rounded to bfloat16, products accumulated in binary32 in
 *           increasing input index, statements summed in increasing s.
 * vscore64: the same network in binary64 with no rounding of inputs or activations (information).
 * vmag:     (may be NULL) sum over the valid statements of  sum_k |w3_k h2_k| + |b3|  on the bfloat16 path: the size of
 *           the terms whose sum vscore is.  One bfloat16 rounding step of an activation is 2^-8 of its size, so two
 *           correct evaluations that round one activation differently differ by about 2^-9 vmag at most, however far
 *           the sum itself cancels: the yardstick for comparing another bfloat16 evaluation with this one.
 */
int orc_verify(const float* feat, const int32_t* n_stmt, int64_t n_d, int32_t max_stmt, int32_t feat_dim, int32_t hidden,
               const uint16_t* W1, const float* b1, const uint16_t* W2, const float* b2, const uint16_t* w3, float b3,
               float* vscore32, double* vscore64, double* vmag)
{
    if (n_d < 0 || max_stmt < 1 || feat_dim < 1 || hidden < 1) return -1;
    float* x = (float*)malloc(sizeof(float) * (size_t)feat_dim);
    float* h1 = (float*)malloc(sizeof(float) * (size_t)hidden);
    float* h2 = (float*)malloc(sizeof(float) * (size_t)hidden);
    double* g1 = (double*)malloc(sizeof(double) * (size_t)hidden);
    double* g2 = (double*)malloc(sizeof(double) * (size_t)hidden);
    if (!x || !h1 || !h2 || !g1 || !g2) return -4;
    int rc = 0;
    for (int64_t c = 0; c < n_d && !rc; ++c) {
        if (n_stmt[c] < 0 || n_stmt[c] > max_stmt) {
            rc = -1;
            break;
        }
        float total = 0.0f;
        double total64 = 0.0, mag = 0.0;
        for (int32_t s = 0; s < n_stmt[c]; ++s) {
            const float* row = feat + ((size_t)c * max_stmt + s) * feat_dim;
            /* bfloat16 path */
            for (int k = 0; k < feat_dim; ++k) x[k] = orc_bf16_round(row[k]);
            for (int o = 0; o < hidden; ++o) {
                float acc = 0.0f;
                for (int k = 0; k < feat_dim; ++k) acc = acc + bf16_bits_to_f32(W1[(size_t)o * feat_dim + k]) * x[k];
                h1[o] = orc_bf16_round(fmaxf(acc + b1[o], 0.0f));
            }
            for (int o = 0; o < hidden; ++o) {
                float acc = 0.0f;
                for (int k = 0; k < hidden; ++k) acc = acc + bf16_bits_to_f32(W2[(size_t)o * hidden + k]) * h1[k];
                h2[o] = orc_bf16_round(fmaxf(acc + b2[o], 0.0f));
            }
            float y = 0.0f;
            for (int k = 0; k < hidden; ++k) y = y + bf16_bits_to_f32(w3[k]) * h2[k];
            y = y + b3;
            total = total + y;
            /* size of what was added up: the yardstick of a comparison in bfloat16 (see vmag above) */
            for (int k = 0; k < hidden; ++k) mag += fabs((double)bf16_bits_to_f32(w3[k]) * (double)h2[k]);
            mag += fabs((double)b3);
            /* binary64 shadow */
            if (vscore64) {
                for (int o = 0; o < hidden; ++o) {
                    double acc = 0.0;
                    for (int k = 0; k < feat_dim; ++k) acc += (double)bf16_bits_to_f32(W1[(size_t)o * feat_dim + k]) * (double)row[k];
                    g1[o] = fmax(acc + (double)b1[o], 0.0);
                }
                for (int o = 0; o < hidden; ++o) {
                    double acc = 0.0;
                    for (int k = 0; k < hidden; ++k) acc += (double)bf16_bits_to_f32(W2[(size_t)o * hidden + k]) * g1[k];
                    g2[o] = fmax(acc + (double)b2[o], 0.0);
                }
                double y64 = 0.0;
                for (int k = 0; k < hidden; ++k) y64 += (double)bf16_bits_to_f32(w3[k]) * g2[k];
                total64 += y64 + (double)b3;
            }
        }
        if (vscore32) vscore32[c] = total;
        if (vscore64) vscore64[c] = total64;
        if (vmag) vmag[c] = mag;
    }
    free(x);
    free(h1);
    free(h2);
    free(g1);
    free(g2);
    return rc;
}

/* ---- latent schedule explorer (Alg. 2): C_SA, PriorFilter and SchMutation over nSteps ---------------------- */

/*
 * Counter-based random numbers: draw c (c >= 1) is the c-th output of SplitMix64 (Steele, Lea, Flood, "Fast
 * splittable pseudorandom number generators", OOPSLA 2014; the public-domain splitmix64.c) started from `seed`.
 */
uint64_t orc_splitmix64_draw(uint64_t seed, uint64_t c)
{
    uint64_t z = seed + c * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* A draw's bit field x of `bits` bits mapped onto 0..n-1: floor(x * n / 2^bits) (no division; n < 2^bits need not hold). */
static uint32_t pick_of(uint64_t x, int bits, uint32_t n) { return (uint32_t)((x * (uint64_t)n) >> bits); }

static int slots_of(const orc_subgraph* sg) { return sg->n_sp * sg->sp_levels + sg->n_rd * sg->rd_levels; }

/*
 * SchMutation of one child (reading: the paper names a genetic algorithm over tiling factors guided by the draft
 * fitness and gives no operator).  Taken here: truncation selection - the parent is one of the k fittest schedules
 * seen so far (S_spec after this step's PriorFilter), chosen uniformly; with probability mutate_q16 / 65536 one
 * prime factor of one tile factor moves to another level of the same axis (the product over the axis is kept), unless
 * that would break a fragment multiple, in which case the child is an unchanged copy.
 * f: the child's factors (already a copy of the parent), stride 1.  u2: the second random draw of this child.
 */
static void mutate_child(const orc_subgraph* sg, uint16_t* f, uint64_t u2)
{
    const int n_axes = sg->n_sp + sg->n_rd;
    const int axis = (int)pick_of(u2 & 0xFF, 8, (uint32_t)n_axes);
    const int levels = axis < sg->n_sp ? sg->sp_levels : sg->rd_levels;
    const int base = axis < sg->n_sp ? axis * sg->sp_levels : sg->n_sp * sg->sp_levels + (axis - sg->n_sp) * sg->rd_levels;
    const int src = (int)pick_of((u2 >> 8) & 0xFF, 8, (uint32_t)levels);
    int dst = (int)pick_of((u2 >> 16) & 0xFF, 8, (uint32_t)(levels - 1));
    if (dst >= src) ++dst;
    const uint32_t v = f[base + src];
    /* distinct prime factors of v, ascending */
    uint32_t primes[16];
    int n_primes = 0;
    uint32_t rest = v;
    for (uint32_t p = 2; p * p <= rest; ++p) {
        if (rest % p == 0) {
            primes[n_primes++] = p;
            while (rest % p == 0) rest /= p;
        }
    }
    if (rest > 1) primes[n_primes++] = rest;
    if (n_primes == 0) return; /* v = 1: nothing to move */
    const uint32_t p = primes[pick_of((u2 >> 24) & 0xFF, 8, (uint32_t)n_primes)];
    if (in_fragment_mode(sg) && src == levels - 1) {
        /* innermost tiles of the last two spatial axes and of the last reduction axis stay whole fragments */
        int frag = 0;
        if (axis == sg->n_sp - 2) frag = sg->frag[0];
        if (axis == sg->n_sp - 1) frag = sg->frag[1];
        if (axis == n_axes - 1) frag = sg->frag[2];
        if (frag > 0 && (v / p) % (uint32_t)frag != 0) return;
    }
    f[base + src] = (uint16_t)(v / p);
    f[base + dst] = (uint16_t)(f[base + dst] * p);
}

/* Identity of a schedule: a 64-bit hash of its tile factors (the subgraph's own slots, in slot order). */
uint64_t orc_schedule_hash(const uint16_t* f, int64_t stride, int n_slots)
{
    uint64_t h = (uint64_t)n_slots;
    for (int r = 0; r < n_slots; ++r) h = orc_splitmix64_draw(h, (uint64_t)f[r * stride] + 1);
    return h;
}

typedef struct {
    float score;
    uint64_t hash;
    int64_t pos; /* place in the union: S_spec's entries first, then the k best of S_x */
} orc_entry;

/* best first: higher score, then smaller hash, then older (smaller position) */
static int by_score_hash_age(const void* pa, const void* pb)
{
    const orc_entry* a = (const orc_entry*)pa;
    const orc_entry* b = (const orc_entry*)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    if (a->hash != b->hash) return a->hash < b->hash ? -1 : 1;
    return (a->pos > b->pos) - (a->pos < b->pos);
}

/*
 * Alg. 2 with the population resident: n_steps times { costs = C_SA(S_x); S_spec = PriorFilter(S_x U S_spec);
 * S_x = SchMutation(S_x, costs) }.
 *   tiles       [rows][pitch] in: the initial S_x (RandomInitSch is the caller's); out: S_x after the last mutation
 *   score       [n] out: C_SA of the last population that was scored (binary32 path)
 *   spec_tiles  [rows][n_sg*k], spec_score [n_sg*k], spec_count [n_sg] out: S_spec, best first; rows a subgraph
 *               does not own and entries past spec_count hold 0 / -infinity
 * PriorFilter, as a procedure (S_x U S_spec is a union of sets: a schedule counts once; the population of a genetic
 * algorithm is full of copies): B = the k best of S_x (score descending, candidate index ascending); U = S_spec
 * followed by B; order U by score descending, schedule hash ascending, position ascending; drop every entry whose
 * score and hash equal its predecessor's; keep the first k of what is left.
 * SchMutation: child j copies S_spec[floor(low32(u1) * spec_count / 2^32)] of its subgraph and mutates it with probability
 * mutate_q16 / 65536 (mutate_child).  Draws of candidate j in step t: counters (t << 41) + 2 j + 1 and + 2.
 * Errors as orc_draft_score and orc_topk; -1 also for n_steps < 1, k < 1, mutate_q16 > 65536.
 */
int orc_lse(const orc_subgraph* sg, int32_t n_sg, const int64_t* seg_off, uint16_t* tiles, int64_t pitch, int32_t rows, int32_t flags,
            int32_t k, int32_t n_steps, uint64_t seed, uint32_t mutate_q16, float* score, uint16_t* spec_tiles, float* spec_score,
            int32_t* spec_count)
{
    if (n_sg <= 0 || k <= 0 || n_steps < 1 || mutate_q16 > 65536) return -1;
    const int64_t spec_pitch = (int64_t)n_sg * k;
    for (int32_t s = 0; s < n_sg; ++s)
        if (seg_off[s + 1] - seg_off[s] < k || slots_of(&sg[s]) > rows) return -1;
    orc_entry* u = (orc_entry*)malloc((size_t)2 * k * sizeof(orc_entry));
    uint16_t* next_tiles = (uint16_t*)malloc((size_t)rows * (size_t)spec_pitch * sizeof(uint16_t));
    float* next_score = (float*)malloc((size_t)spec_pitch * sizeof(float));
    int32_t* best = (int32_t*)malloc((size_t)spec_pitch * sizeof(int32_t));
    float* best_val = (float*)malloc((size_t)spec_pitch * sizeof(float));
    if (!u || !next_tiles || !next_score || !best || !best_val) {
        free(u), free(next_tiles), free(next_score), free(best), free(best_val);
        return -4;
    }
    memset(spec_tiles, 0, (size_t)rows * (size_t)spec_pitch * sizeof(uint16_t));
    for (int32_t s = 0; s < n_sg; ++s) spec_count[s] = 0;
    int rc = 0;
    for (int32_t t = 0; t < n_steps && !rc; ++t) {
        rc = orc_draft_score(sg, n_sg, seg_off, tiles, pitch, flags, score, NULL, NULL);
        if (!rc) rc = orc_topk(score, seg_off, n_sg, k, best, best_val);
        if (rc) break;
        memset(next_tiles, 0, (size_t)rows * (size_t)spec_pitch * sizeof(uint16_t));
        for (int32_t s = 0; s < n_sg; ++s) {
            const int n_slots = slots_of(&sg[s]);
            const int64_t col0 = (int64_t)s * k, n_old = spec_count[s];
            for (int64_t i = 0; i < n_old; ++i) {
                u[i].score = spec_score[col0 + i];
                u[i].hash = orc_schedule_hash(spec_tiles + col0 + i, spec_pitch, n_slots);
                u[i].pos = i;
            }
            for (int64_t r = 0; r < k; ++r) {
                u[n_old + r].score = best_val[col0 + r];
                u[n_old + r].hash = orc_schedule_hash(tiles + best[col0 + r], pitch, n_slots);
                u[n_old + r].pos = n_old + r;
            }
            qsort(u, (size_t)(n_old + k), sizeof(orc_entry), by_score_hash_age);
            int32_t kept = 0;
            for (int64_t i = 0; i < n_old + k && kept < k; ++i) {
                if (i > 0 && u[i].score == u[i - 1].score && u[i].hash == u[i - 1].hash) continue; /* a copy */
                const int64_t pos = u[i].pos;
                next_score[col0 + kept] = u[i].score;
                for (int row = 0; row < n_slots; ++row)
                    next_tiles[row * spec_pitch + col0 + kept] = pos < n_old ? spec_tiles[row * spec_pitch + col0 + pos]
                                                                             : tiles[row * pitch + best[col0 + (pos - n_old)]];
                ++kept;
            }
            for (int32_t r = kept; r < k; ++r) next_score[col0 + r] = -INFINITY;
            spec_count[s] = kept;
        }
        memcpy(spec_tiles, next_tiles, (size_t)rows * (size_t)spec_pitch * sizeof(uint16_t));
        memcpy(spec_score, next_score, (size_t)spec_pitch * sizeof(float));
        for (int32_t s = 0; s < n_sg; ++s) {
            const int n_slots = slots_of(&sg[s]);
            for (int64_t j = seg_off[s]; j < seg_off[s + 1]; ++j) {
                const uint64_t c = ((uint64_t)t << 41) + 2 * (uint64_t)j;
                const uint64_t u1 = orc_splitmix64_draw(seed, c + 1), u2 = orc_splitmix64_draw(seed, c + 2);
                const int64_t parent = (int64_t)s * k + (int64_t)pick_of(u1 & 0xFFFFFFFFu, 32, (uint32_t)spec_count[s]);
                uint16_t child[ORC_MAX_AXES * 4];
                for (int row = 0; row < n_slots; ++row) child[row] = spec_tiles[row * spec_pitch + parent];
                if (((u1 >> 32) & 0xFFFF) < mutate_q16) mutate_child(&sg[s], child, u2);
                for (int row = 0; row < n_slots; ++row) tiles[row * pitch + j] = child[row];
            }
        }
    }
    free(u), free(next_tiles), free(next_score), free(best), free(best_val);
    return rc;
}

/* ------------------------------------------------------------------------------------------------------------------
 * RandomInitSch (Alg. 1: S_draft = S_spec U RandomInitSch(p0); Alg. 2: the initial S_x): schedules drawn uniformly
 * from the schedule space.  The paper says "randomly samples" and no more; the reading taken here:
 *   - a schedule is one ordered factorisation of every axis extent into the axis's levels (4 spatial, 2 or 3
 *     reduction), all axes independent; in fragment mode the innermost factor of the last two spatial axes and of
 *     the last reduction axis is a multiple of the fragment size g: factorise extent / g and multiply the innermost
 *     factor by g;
 *   - the ordered L-factorisations of b = p1^e1 p2^e2 ... (primes ascending) are the tuples of weak compositions of
 *     e1, e2, ... into L parts: part l of the composition of e_i is the exponent of p_i in the factor of level l
 *     (outermost level first).  A composition's number is its rank in lexicographic order of (x_0, ..., x_{L-1});
 *     a factorisation's number is R = r_1 + C_1 (r_2 + C_2 (r_3 + ...)), C_i = binom(e_i + L - 1, L - 1);
 *   - candidate c (global index), axis a: R = floor(u * count / 2^64), u = draw number 8 c + a + 1 of SplitMix64
 *     started from `seed`, count = product of the C_i.
 * Returns 0, or -1 if an extent is not a multiple of its fragment size or a factor would not fit 16 bits.
 */
static uint64_t binom_small(int n, int k)
{
    if (k < 0 || k > n) return 0;
    uint64_t r = 1;
    for (int i = 1; i <= k; ++i) r = r * (uint64_t)(n - k + i) / (uint64_t)i; /* exact at every step */
    return r;
}

/* the composition of e into `levels` parts with lexicographic rank r */
static void unrank_composition(int e, int levels, uint64_t r, int* x)
{
    int rest = e;
    for (int l = 0; l < levels - 1; ++l) {
        const int parts_left = levels - l - 1; /* parts after this one */
        int v = 0;
        for (;; ++v) {
            const uint64_t cnt = binom_small(rest - v + parts_left - 1, parts_left - 1); /* compositions of rest - v into parts_left parts */
            if (r < cnt) break;
            r -= cnt;
        }
        x[l] = v;
        rest -= v;
    }
    x[levels - 1] = rest;
}

static int axis_fragment(const orc_subgraph* sg, int axis)
{
    if (!in_fragment_mode(sg)) return 1;
    if (axis == sg->n_sp - 2) return sg->frag[0];
    if (axis == sg->n_sp - 1) return sg->frag[1];
    if (axis == sg->n_sp + sg->n_rd - 1) return sg->frag[2];
    return 1;
}

/* number of ordered factorisations of the axis (after taking out the fragment); 0 if the fragment does not divide it */
uint64_t orc_axis_space(const orc_subgraph* sg, int axis)
{
    const int levels = axis < sg->n_sp ? sg->sp_levels : sg->rd_levels;
    const int g = axis_fragment(sg, axis);
    if (sg->extent[axis] % g != 0) return 0;
    uint32_t rest = (uint32_t)(sg->extent[axis] / g);
    uint64_t count = 1;
    for (uint32_t p = 2; p * p <= rest; ++p) {
        int e = 0;
        while (rest % p == 0) rest /= p, ++e;
        if (e) count *= binom_small(e + levels - 1, levels - 1);
    }
    if (rest > 1) count *= (uint64_t)levels;
    return count;
}

int orc_random_init(const orc_subgraph* sg, int32_t n_sg, const int64_t* seg_off, uint16_t* tiles, int64_t pitch, uint64_t seed)
{
    for (int s = 0; s < n_sg; ++s) {
        const orc_subgraph* g = &sg[s];
        const int n_axes = g->n_sp + g->n_rd;
        for (int a = 0; a < n_axes; ++a)
            if (orc_axis_space(g, a) == 0) return -1;
        for (int64_t c = seg_off[s]; c < seg_off[s + 1]; ++c) {
            int slot = 0;
            for (int a = 0; a < n_axes; ++a) {
                const int levels = a < g->n_sp ? g->sp_levels : g->rd_levels;
                const int frag = axis_fragment(g, a);
                const uint64_t count = orc_axis_space(g, a);
                const uint64_t u = orc_splitmix64_draw(seed, 8 * (uint64_t)c + (uint64_t)a + 1);
                uint64_t R = (uint64_t)(((unsigned __int128)u * count) >> 64);
                uint32_t f[4] = {1, 1, 1, 1};
                uint32_t rest = (uint32_t)(g->extent[a] / frag);
                for (uint32_t p = 2; rest > 1; ++p) {
                    if (p * p > rest) p = rest; /* what is left is prime */
                    int e = 0;
                    while (rest % p == 0) rest /= p, ++e;
                    if (!e) continue;
                    const uint64_t C = binom_small(e + levels - 1, levels - 1);
                    int x[4];
                    unrank_composition(e, levels, R % C, x);
                    R /= C;
                    for (int l = 0; l < levels; ++l)
                        for (int i = 0; i < x[l]; ++i) f[l] *= p;
                }
                f[levels - 1] *= (uint32_t)frag;
                for (int l = 0; l < levels; ++l) {
                    if (f[l] > 65535u) return -1;
                    tiles[(int64_t)(slot + l) * pitch + c] = (uint16_t)f[l];
                }
                slot += levels;
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------------------------------
 * Momentum online Adaptation (Sec. 4.3; Alg. 1's Update_MoA; momentum m = 0.99 in the figure's caption).  Each round
 * the target model starts from the Siamese model's weights phi_s and is fine-tuned on the records collected online
 * (that training is not part of this path); then the Siamese weights follow the target's, as in momentum contrast:
 *     phi_s <- m phi_s + (1 - m) phi_t
 * (with phi_t = phi_s - lr * sum of the target's gradients this is phi_s - (1 - m) lr * sum Delta_t: the update "according
 * to the gradients of the target model", with no forward or backward pass of the Siamese model).  The paper's formula
 * sits in a figure that is lost; this is the reading taken.
 * binary32, in this order, each operation rounded: c = 1 - m;  phi_s = (m * phi_s) + (c * phi_t).
 * out64 (optional) receives the same in binary64 from the binary32 inputs; bf16 (optional) the new phi_s rounded to
 * bfloat16 (nearest, ties to even): the copy the verify stage reads.
 */
int orc_moa_update(float* phi_s, const float* phi_t, int64_t n, float m, uint16_t* bf16, double* out64)
{
    if (!phi_s || !phi_t || n < 0 || !(m >= 0.0f && m <= 1.0f)) return -1;
    const float c = 1.0f - m;
    for (int64_t i = 0; i < n; ++i) {
        if (out64) out64[i] = (double)m * (double)phi_s[i] + (1.0 - (double)m) * (double)phi_t[i];
        const float a = m * phi_s[i];
        const float b = c * phi_t[i];
        const float v = a + b;
        phi_s[i] = v;
        if (bf16) {
            const float r = orc_bf16_round(v);
            uint32_t u;
            memcpy(&u, &r, 4);
            bf16[i] = (uint16_t)(u >> 16);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------------------------------
 * The whole Pattern-aware Transformer (Sec. 4.2): a statement branch ("multiple linear layers, followed by summation
 * to obtain a high-dimension vector"), a temporal-dataflow branch ("a self-attention mechanism to model context
 * dependencies" over 23-dimensional data-block features), and a head ("a concatenation operator and multiple linear
 * layers").  The figure with the dimensions is lost; the reading taken (hidden 256, embedding 64, one attention head, one
 * attention layer with a residual connection, sum pooling, one hidden head layer):
 *   statement s < n_stmt:  h1 = relu(W1 x_s + b1);  h2 = relu(W2 h1 + b2);          v_s = sum_s h2          (256)
 *   block i < n_blk:       e_i = relu(We d_i + be);  q_i, k_i, v_i = Wq e_i, Wk e_i, Wv e_i
 *                          a_ij = softmax_j(q_i . k_j / sqrt(64)),  o_i = sum_j a_ij v_j
 *                          z_i = e_i + Wo o_i;                                     v_d = sum_i z_i         (64)
 *   head:                  g = relu(Wh [v_s ; v_d] + bh);  y = wo . g + bo
 * A candidate without data blocks (an element-wise operator; the paper pads its features with zeros) has v_d = 0.
 * Precision as in orc_verify: every operand of a matrix product is rounded to bfloat16 (inputs, e, q, k, v, o, h1, h2,
 * and the head's input), products are accumulated in binary32 in increasing input index, sums over statements and
 * blocks in increasing index, the softmax in binary32 (expf of the score minus the row maximum).
 * y64: the same network in binary64 without any rounding (information).
 */
typedef struct {
    const uint16_t *W1, *W2;          /* [256][164], [256][256] */
    const float *b1, *b2;
    const uint16_t *We;               /* [64][23] */
    const float* be;
    const uint16_t *Wq, *Wk, *Wv, *Wo; /* [64][64] each */
    const uint16_t* Wh;               /* [256][320] */
    const float* bh;
    const uint16_t* wo;               /* [256] */
    float bo;
} orc_pacm_weights;

#define PACM_F 164
#define PACM_H 256
#define PACM_D 23
#define PACM_E 64
#define PACM_T 8

static void matvec_bf16(const uint16_t* W, int rows, int cols, const float* x, const float* bias, float* out)
{
    for (int o = 0; o < rows; ++o) {
        float acc = 0.0f;
        for (int k = 0; k < cols; ++k) acc = acc + bf16_bits_to_f32(W[(size_t)o * cols + k]) * x[k];
        out[o] = bias ? acc + bias[o] : acc;
    }
}

static void matvec_f64(const uint16_t* W, int rows, int cols, const double* x, const float* bias, double* out)
{
    for (int o = 0; o < rows; ++o) {
        double acc = 0.0;
        for (int k = 0; k < cols; ++k) acc += (double)bf16_bits_to_f32(W[(size_t)o * cols + k]) * x[k];
        out[o] = bias ? acc + (double)bias[o] : acc;
    }
}

int orc_pacm(const float* feat, const int32_t* n_stmt, const float* flow, const int32_t* n_blk, int64_t n_d, const orc_pacm_weights* w,
             float* y32, double* y64)
{
    if (n_d < 0 || !w) return -1;
    for (int64_t c = 0; c < n_d; ++c) {
        if (n_stmt[c] < 0 || n_stmt[c] > PACM_T || n_blk[c] < 0 || n_blk[c] > PACM_T) return -1;
        /* ---- bfloat16 path ---- */
        float vs[PACM_H], vd[PACM_E];
        for (int h = 0; h < PACM_H; ++h) vs[h] = 0.0f;
        for (int e = 0; e < PACM_E; ++e) vd[e] = 0.0f;
        for (int s = 0; s < n_stmt[c]; ++s) {
            float x[PACM_F], h1[PACM_H], h2[PACM_H];
            const float* row = feat + ((size_t)c * PACM_T + s) * PACM_F;
            for (int k = 0; k < PACM_F; ++k) x[k] = orc_bf16_round(row[k]);
            matvec_bf16(w->W1, PACM_H, PACM_F, x, w->b1, h1);
            for (int h = 0; h < PACM_H; ++h) h1[h] = orc_bf16_round(fmaxf(h1[h], 0.0f));
            matvec_bf16(w->W2, PACM_H, PACM_H, h1, w->b2, h2);
            for (int h = 0; h < PACM_H; ++h) vs[h] = vs[h] + orc_bf16_round(fmaxf(h2[h], 0.0f));
        }
        const int T = n_blk[c];
        float e[PACM_T][PACM_E], q[PACM_T][PACM_E], k[PACM_T][PACM_E], v[PACM_T][PACM_E];
        for (int i = 0; i < T; ++i) {
            float d[PACM_D];
            const float* row = flow + ((size_t)c * PACM_T + i) * PACM_D;
            for (int j = 0; j < PACM_D; ++j) d[j] = orc_bf16_round(row[j]);
            matvec_bf16(w->We, PACM_E, PACM_D, d, w->be, e[i]);
            for (int j = 0; j < PACM_E; ++j) e[i][j] = orc_bf16_round(fmaxf(e[i][j], 0.0f));
            matvec_bf16(w->Wq, PACM_E, PACM_E, e[i], NULL, q[i]);
            matvec_bf16(w->Wk, PACM_E, PACM_E, e[i], NULL, k[i]);
            matvec_bf16(w->Wv, PACM_E, PACM_E, e[i], NULL, v[i]);
            for (int j = 0; j < PACM_E; ++j) q[i][j] = orc_bf16_round(q[i][j]), k[i][j] = orc_bf16_round(k[i][j]), v[i][j] = orc_bf16_round(v[i][j]);
        }
        for (int i = 0; i < T; ++i) {
            float sc[PACM_T], mx = -INFINITY, den = 0.0f, o[PACM_E], z[PACM_E];
            for (int j = 0; j < T; ++j) {
                float acc = 0.0f;
                for (int t = 0; t < PACM_E; ++t) acc = acc + q[i][t] * k[j][t];
                sc[j] = acc * 0.125f;
                mx = fmaxf(mx, sc[j]);
            }
            for (int j = 0; j < T; ++j) sc[j] = expf(sc[j] - mx), den = den + sc[j];
            for (int t = 0; t < PACM_E; ++t) {
                float acc = 0.0f;
                for (int j = 0; j < T; ++j) acc = acc + (sc[j] / den) * v[j][t];
                o[t] = orc_bf16_round(acc);
            }
            matvec_bf16(w->Wo, PACM_E, PACM_E, o, NULL, z);
            for (int t = 0; t < PACM_E; ++t) vd[t] = vd[t] + (e[i][t] + z[t]);
        }
        float u[PACM_H + PACM_E], g[PACM_H];
        for (int h = 0; h < PACM_H; ++h) u[h] = orc_bf16_round(vs[h]);
        for (int t = 0; t < PACM_E; ++t) u[PACM_H + t] = orc_bf16_round(vd[t]);
        matvec_bf16(w->Wh, PACM_H, PACM_H + PACM_E, u, w->bh, g);
        float y = 0.0f;
        for (int h = 0; h < PACM_H; ++h) y = y + bf16_bits_to_f32(w->wo[h]) * orc_bf16_round(fmaxf(g[h], 0.0f));
        y32[c] = y + w->bo;
        /* ---- binary64 shadow ---- */
        if (y64) {
            double VS[PACM_H], VD[PACM_E];
            for (int h = 0; h < PACM_H; ++h) VS[h] = 0.0;
            for (int t = 0; t < PACM_E; ++t) VD[t] = 0.0;
            for (int s = 0; s < n_stmt[c]; ++s) {
                double x[PACM_F], h1[PACM_H], h2[PACM_H];
                const float* row = feat + ((size_t)c * PACM_T + s) * PACM_F;
                for (int kk = 0; kk < PACM_F; ++kk) x[kk] = (double)row[kk];
                matvec_f64(w->W1, PACM_H, PACM_F, x, w->b1, h1);
                for (int h = 0; h < PACM_H; ++h) h1[h] = h1[h] > 0.0 ? h1[h] : 0.0;
                matvec_f64(w->W2, PACM_H, PACM_H, h1, w->b2, h2);
                for (int h = 0; h < PACM_H; ++h) VS[h] += h2[h] > 0.0 ? h2[h] : 0.0;
            }
            double E[PACM_T][PACM_E], Q[PACM_T][PACM_E], K[PACM_T][PACM_E], V[PACM_T][PACM_E];
            for (int i = 0; i < T; ++i) {
                double d[PACM_D];
                const float* row = flow + ((size_t)c * PACM_T + i) * PACM_D;
                for (int j = 0; j < PACM_D; ++j) d[j] = (double)row[j];
                matvec_f64(w->We, PACM_E, PACM_D, d, w->be, E[i]);
                for (int j = 0; j < PACM_E; ++j) E[i][j] = E[i][j] > 0.0 ? E[i][j] : 0.0;
                matvec_f64(w->Wq, PACM_E, PACM_E, E[i], NULL, Q[i]);
                matvec_f64(w->Wk, PACM_E, PACM_E, E[i], NULL, K[i]);
                matvec_f64(w->Wv, PACM_E, PACM_E, E[i], NULL, V[i]);
            }
            for (int i = 0; i < T; ++i) {
                double sc[PACM_T], mx = -INFINITY, den = 0.0, o[PACM_E], z[PACM_E];
                for (int j = 0; j < T; ++j) {
                    double acc = 0.0;
                    for (int t = 0; t < PACM_E; ++t) acc += Q[i][t] * K[j][t];
                    sc[j] = acc * 0.125;
                    mx = sc[j] > mx ? sc[j] : mx;
                }
                for (int j = 0; j < T; ++j) sc[j] = exp(sc[j] - mx), den += sc[j];
                for (int t = 0; t < PACM_E; ++t) {
                    double acc = 0.0;
                    for (int j = 0; j < T; ++j) acc += (sc[j] / den) * V[j][t];
                    o[t] = acc;
                }
                matvec_f64(w->Wo, PACM_E, PACM_E, o, NULL, z);
                for (int t = 0; t < PACM_E; ++t) VD[t] += E[i][t] + z[t];
            }
            double U[PACM_H + PACM_E], G[PACM_H], Y = 0.0;
            for (int h = 0; h < PACM_H; ++h) U[h] = VS[h];
            for (int t = 0; t < PACM_E; ++t) U[PACM_H + t] = VD[t];
            matvec_f64(w->Wh, PACM_H, PACM_H + PACM_E, U, w->bh, G);
            for (int h = 0; h < PACM_H; ++h) Y += (double)bf16_bits_to_f32(w->wo[h]) * (G[h] > 0.0 ? G[h] : 0.0);
            y64[c] = Y + (double)w->bo;
        }
    }
    return 0;
}
