/*
 * CPU oracle for the OSP synchronization step.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain, slow, by-eye-checkable statement of what one OSP
 * iteration computes on the parameter-server side and on each worker.  It is
 * independent of the HIP library: no shared headers, helpers, tables or
 * constants.  Only the tests, the smoke check and the benchmark's CPU-baseline
 * leg may load it; the product never does.
 *
 * Every function is the definition written out as loops over tensors and
 * elements, one IEEE-754 binary32 operation per C operator (build with
 * -ffp-contract=off, no fast-math), in the paper's order:
 *
 *   aggregate  Sec. 2.1.1 : PS weights each worker's gradient by its data
 *                           share, merges, updates the global parameters.
 *   PGP        Sec. 4.1.1, I_k = |G_k P_k| (text after Eq. 3), Eq. 4 per layer.
 *   split      Sec. 4.1.1-4.1.2: rank by importance, send the least important
 *                           S(G^u) to the in-computation stage.
 *   LGP        Sec. 4.2, Eq. 6: stale stage-2 parameters advance by the
 *                           worker's own local gradient.
 *   correction Sec. 4.2, Eq. 7: the local estimate is replaced by the global
 *                           result once stage 2 has been synchronized.
 *   splitter   Sec. 4.5   : a worker's gradient cut by the GIB into the dense
 *                           arrays G^i and G^u, and the PS update fed by them.
 *
 * Readings taken where the paper is silent (each also listed in the design
 * document): sequential fp32 summation over workers in ascending index;
 * SGD with momentum in the form V <- mu V + g, P <- P - lr V; the PGP product
 * uses the aggregated gradient and the PS parameter before this update;
 * NaN magnitudes are canonicalised so they compare equal and above +Inf;
 * ties in every ranking break by ascending index; GIB polarity 1 = important
 * (stage 1, routine synchronization).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * against closed forms, a NumPy brute force, torch.optim.SGD and the
 * invariants the paper states (Sec. 4.3 degradation to BSP / ASP; Sec. 2.2.2
 * and 3.2: OSP discards no gradient).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { OSP_ORACLE_GRAN_LAYER = 0, OSP_ORACLE_GRAN_ELEMENT = 1 };

typedef struct {
    int32_t n_workers;           /* N */
    int32_t n_tensors;           /* L */
    const int64_t *numel;        /* [L] */
    const int64_t *offset;       /* [L] element offsets into every arena */
    int64_t arena_elems;
    float lr;
    float momentum;
    const float *worker_weight;  /* [N] data shares, or NULL for 1/N each */
} osp_oracle_model;

/* Gradient Importance Bitmap (Sec. 3.2): 1 = important = stage 1 (RS),
 * 0 = unimportant = stage 2 (ICS).  One byte per layer, or one bit per arena
 * element (bit k%32 of word k/32). */
typedef struct {
    int32_t granularity;
    const uint8_t *layer;        /* [L]            when granularity == LAYER   */
    const uint32_t *bits;        /* [ceil(arena/32)] when granularity == ELEMENT */
} osp_oracle_gib;

static int stage_of(const osp_oracle_gib *gib, int32_t l, int64_t k)
{
    int important;
    if (gib->granularity == OSP_ORACLE_GRAN_LAYER)
        important = gib->layer[l] != 0;
    else
        important = (int)((gib->bits[k >> 5] >> (k & 31)) & 1u);
    return important ? 1 : 2;
}

/* stage: 1 or 2 = only that stage's elements; 0 = every element (a plain BSP
 * step, Sec. 4.3).  gib may be NULL when stage == 0. */
static int selected(const osp_oracle_gib *gib, int stage, int32_t l, int64_t k)
{
    return stage == 0 || stage_of(gib, l, k) == stage;
}

/* The aggregate of one element (Sec. 2.1.1): the workers' gradients weighted
 * by their data shares and merged, sequentially in ascending worker order;
 * with equal shares the plain sum times fl(1/N).  g points at worker 0's value,
 * worker w's is stride elements further on. */
static float aggregate_element(const osp_oracle_model *m, const float *g, int64_t stride)
{
    const int N = m->n_workers;
    const float inv_n = 1.0f / (float)N;
    float gbar;
    if (m->worker_weight) {
        float acc = m->worker_weight[0] * g[0];
        for (int w = 1; w < N; ++w) {
            float term = m->worker_weight[w] * g[(int64_t)w * stride];
            acc = acc + term;
        }
        gbar = acc;
    } else {
        float acc = g[0];
        for (int w = 1; w < N; ++w)
            acc = acc + g[(int64_t)w * stride];
        gbar = acc * inv_n;
    }
    return gbar;
}

/* PGP product with the parameter before the update (text after Eq. 3), then
 * SGD with momentum on the PS. */
static void update_element(const osp_oracle_model *m, float gbar, float *P, float *V, float *q,
                           int64_t k)
{
    float prod = gbar * P[k];
    q[k] = fabsf(prod);
    float mv = m->momentum * V[k];
    float v = mv + gbar;
    float step = m->lr * v;
    V[k] = v;
    P[k] = P[k] - step;
}

/*
 * PS side of one stage (Sec. 2.1.1; per stage as in Sec. 3.1).
 * For every element k of the stage:
 *     gbar = sum_w alpha_w g_{w,k}                      (aggregate)
 *     q_k  = |gbar * P_k|                               (PGP, with P before the update)
 *     V_k  = mu V_k + gbar ;  P_k = P_k - lr V_k        (SGD with momentum)
 * q is an [arena] output; entries outside the stage are left as they were.
 */
void osp_oracle_aggregate_update(const osp_oracle_model *m, const osp_oracle_gib *gib,
                                 int stage, float *P, float *V, const float *grads,
                                 int64_t worker_stride, float *q)
{
    for (int32_t l = 0; l < m->n_tensors; ++l) {
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
        for (int64_t j = 0; j < m->numel[l]; ++j) {
            const int64_t k = m->offset[l] + j;
            if (!selected(gib, stage, l, k))
                continue;
            update_element(m, aggregate_element(m, grads + k, worker_stride), P, V, q, k);
        }
    }
}

/* Workers receive the stage's global parameters (Sec. 2.1.1; for stage 2 this
 * is the correction of Eq. 7 taken as an overwrite). */
void osp_oracle_apply_stage(const osp_oracle_model *m, const osp_oracle_gib *gib, int stage,
                            const float *P, float *Pw, int64_t param_stride)
{
    for (int w = 0; w < m->n_workers; ++w)
        for (int32_t l = 0; l < m->n_tensors; ++l) {
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
            for (int64_t j = 0; j < m->numel[l]; ++j) {
                const int64_t k = m->offset[l] + j;
                if (selected(gib, stage, l, k))
                    Pw[(int64_t)w * param_stride + k] = P[k];
            }
        }
}

/* LGP (Eq. 6): each worker moves its stale stage-2 parameters by its own
 * local gradient, P_{w,k} <- P_{w,k} - lr g_{w,k}; no momentum locally. */
void osp_oracle_lgp_correct(const osp_oracle_model *m, const osp_oracle_gib *gib,
                            float *Pw, int64_t param_stride,
                            const float *grads, int64_t worker_stride)
{
    for (int w = 0; w < m->n_workers; ++w)
        for (int32_t l = 0; l < m->n_tensors; ++l) {
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
            for (int64_t j = 0; j < m->numel[l]; ++j) {
                const int64_t k = m->offset[l] + j;
                if (stage_of(gib, l, k) != 2)
                    continue;
                float step = m->lr * grads[(int64_t)w * worker_stride + k];
                float *p = &Pw[(int64_t)w * param_stride + k];
                *p = *p - step;
            }
        }
}

/*
 * Gradient splitter (Sec. 4.5): a worker separates its local gradient,
 * according to the GIB, into the important gradients G^i (stage 1) and the
 * unimportant gradients G^u (stage 2).  Each part is dense: the elements of its
 * stage in arena order, nothing in between.  g is ONE worker's arena; g_i and
 * g_u may each be NULL.  Returns the number of elements of G^u.
 */
int64_t osp_oracle_split_gradients(const osp_oracle_model *m, const osp_oracle_gib *gib,
                                   const float *g, float *g_i, float *g_u)
{
    int64_t n_i = 0, n_u = 0;
    for (int32_t l = 0; l < m->n_tensors; ++l)
        for (int64_t j = 0; j < m->numel[l]; ++j) {
            const int64_t k = m->offset[l] + j;
            if (stage_of(gib, l, k) == 1) {
                if (g_i)
                    g_i[n_i] = g[k];
                ++n_i;
            } else {
                if (g_u)
                    g_u[n_u] = g[k];
                ++n_u;
            }
        }
    return n_u;
}

/*
 * PS side of one stage when the stage's gradients arrive in the dense form
 * above (worker w's part at packed + w * packed_stride): the same aggregate,
 * PGP product and update as osp_oracle_aggregate_update, element i of the
 * dense arrays belonging to the i-th element of the stage in arena order.
 */
void osp_oracle_aggregate_update_packed(const osp_oracle_model *m, const osp_oracle_gib *gib,
                                        int stage, float *P, float *V, const float *packed,
                                        int64_t packed_stride, float *q)
{
    int64_t i = 0;
    for (int32_t l = 0; l < m->n_tensors; ++l)
        for (int64_t j = 0; j < m->numel[l]; ++j) {
            const int64_t k = m->offset[l] + j;
            if (stage_of(gib, l, k) != stage)
                continue;
            update_element(m, aggregate_element(m, packed + i, packed_stride), P, V, q, k);
            ++i;
        }
}

/* Eq. 7 taken literally, in fp64, for stage-2 elements:
 *     P_w <- P_w - G^l + G^g,  G^l = -lr g_w (what LGP added),
 *                              G^g = P_new - P_old (what the PS added).
 * Used only to show that it agrees with the overwrite above. */
void osp_oracle_eq7_literal(const osp_oracle_model *m, const osp_oracle_gib *gib,
                            const float *Pw, int64_t param_stride,
                            const float *grads, int64_t worker_stride,
                            const float *P_old, const float *P_new, double *out)
{
    for (int w = 0; w < m->n_workers; ++w)
        for (int32_t l = 0; l < m->n_tensors; ++l)
            for (int64_t j = 0; j < m->numel[l]; ++j) {
                const int64_t k = m->offset[l] + j;
                const int64_t i = (int64_t)w * param_stride + k;
                if (stage_of(gib, l, k) != 2) {
                    out[i] = (double)Pw[i];
                    continue;
                }
                double g_local = -(double)m->lr * (double)grads[(int64_t)w * worker_stride + k];
                double g_global = (double)P_new[k] - (double)P_old[k];
                out[i] = (double)Pw[i] - g_local + g_global;
            }
}

/* Eq. 4: I^l = sum_{j in l} |g_j P_j|, accumulated in fp64 with Neumaier's
 * compensated summation in index order. */
void osp_oracle_layer_importance(const osp_oracle_model *m, const float *q, double *imp)
{
    for (int32_t l = 0; l < m->n_tensors; ++l) {
        double sum = 0.0, comp = 0.0;
        for (int64_t j = 0; j < m->numel[l]; ++j) {
            double x = (double)q[m->offset[l] + j];
            double t = sum + x;
            if (isfinite(t)) {
                if (fabs(sum) >= fabs(x))
                    comp += (sum - t) + x;
                else
                    comp += (x - t) + sum;
            }
            sum = t;
        }
        imp[l] = isfinite(sum) ? sum + comp : sum;
    }
}

/* total order on importances: NaN is the largest value, all NaNs are equal */
static int imp_less(double a, int32_t ia, double b, int32_t ib)
{
    int na = isnan(a), nb = isnan(b);
    if (na || nb) {
        if (na != nb)
            return nb;             /* a < b iff only b is NaN */
        return ia < ib;
    }
    if (a != b)
        return a < b;
    return ia < ib;
}

/*
 * Layer-granular split (Sec. 4.1.1-4.1.2): rank layers by (I^l, l) ascending;
 * stage 2 is the longest prefix of that ranking whose total size stays within
 * budget_elems.  gib_out[l] = 0 for stage-2 layers, 1 otherwise.  order_out
 * (may be NULL) receives the ranking.  Returns the number of stage-2 elements.
 */
int64_t osp_oracle_split_layer(const osp_oracle_model *m, const double *imp,
                               int64_t budget_elems, uint8_t *gib_out, int32_t *order_out)
{
    const int32_t L = m->n_tensors;
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
    for (int32_t i = 0; i < L; ++i)
        order[i] = i;
    for (int32_t i = 1; i < L; ++i) {        /* insertion sort on the total order */
        int32_t cur = order[i];
        int32_t j = i;
        while (j > 0 && imp_less(imp[cur], cur, imp[order[j - 1]], order[j - 1])) {
            order[j] = order[j - 1];
            --j;
        }
        order[j] = cur;
    }
    for (int32_t l = 0; l < L; ++l)
        gib_out[l] = 1;
    int64_t taken = 0;
    for (int32_t r = 0; r < L; ++r) {
        int32_t l = order[r];
        if (taken + m->numel[l] > budget_elems)
            break;                           /* prefix rule: stop at the first misfit */
        taken += m->numel[l];
        gib_out[l] = 0;
    }
    if (order_out)
        memcpy(order_out, order, sizeof(int32_t) * (size_t)L);
    free(order);
    return taken;
}

/* Selection key of one element: the bit pattern of the non-negative fp32
 * magnitude |g P|; unsigned comparison of keys equals numeric comparison,
 * with +Inf above every finite value and the one canonical NaN above +Inf. */
static uint32_t key_of(float q)
{
    uint32_t u;
    if (isnan(q))
        return 0x7FC00000u;
    memcpy(&u, &q, sizeof u);
    return u & 0x7FFFFFFFu;
}

void osp_oracle_keys(const osp_oracle_model *m, const float *q, uint32_t *key)
{
    for (int32_t l = 0; l < m->n_tensors; ++l)
        for (int64_t j = 0; j < m->numel[l]; ++j) {
            const int64_t k = m->offset[l] + j;
            key[k] = key_of(q[k]);
        }
}

typedef struct { uint32_t key; int64_t index; } key_index;

static int cmp_key_index(const void *a, const void *b)
{
    const key_index *x = (const key_index *)a, *y = (const key_index *)b;
    if (x->key != y->key)
        return x->key < y->key ? -1 : 1;
    if (x->index != y->index)
        return x->index < y->index ? -1 : 1;
    return 0;
}

/*
 * Element-granular split: stage 2 is the budget_elems elements that come first
 * in the order (I_k ascending, arena index ascending), I_k = |G_k P_k|.
 * bits_out gets one bit per arena element, 1 = important; padding bits are 1.
 * Returns the number of stage-2 elements (= budget_elems), or -1 if the
 * budget is outside [0, number of parameters].
 */
int64_t osp_oracle_split_element(const osp_oracle_model *m, const float *q,
                                 int64_t budget_elems, uint32_t *bits_out)
{
    int64_t total = 0;
    for (int32_t l = 0; l < m->n_tensors; ++l)
        total += m->numel[l];
    if (budget_elems < 0 || budget_elems > total)
        return -1;
    key_index *a = (key_index *)malloc(sizeof(key_index) * (size_t)(total > 0 ? total : 1));
    int64_t n = 0;
    for (int32_t l = 0; l < m->n_tensors; ++l)
        for (int64_t j = 0; j < m->numel[l]; ++j) {
            const int64_t k = m->offset[l] + j;
            a[n].key = key_of(q[k]);
            a[n].index = k;
            ++n;
        }
    qsort(a, (size_t)n, sizeof(key_index), cmp_key_index);
    const int64_t words = (m->arena_elems + 31) / 32;
    for (int64_t i = 0; i < words; ++i)
        bits_out[i] = 0xFFFFFFFFu;
    for (int64_t r = 0; r < budget_elems; ++r) {
        const int64_t k = a[r].index;
        bits_out[k >> 5] &= ~(1u << (k & 31));
    }
    free(a);
    return budget_elems;
}

/*
 * S(G^u) tuning.  Eq. 5: the in-computation stage must fit into the compute
 * time of one iteration, T_c >= N S(G^u) / (b (1 + lr)), lr being the loss rate
 * of the link, hence U_max = b (1 + lr) T_c / N (taken as printed).
 */
double osp_oracle_ics_upper_bound(double b, double loss_rate, double t_c, int n_workers)
{
    return b * (1.0 + loss_rate) * t_c / (double)n_workers;
}

/*
 * Algorithm 1, one epoch of it: U_max is limited to 80 % of the model size; in
 * epoch 1 everything is synchronized in stage 1 (S = 0) and the loss of that
 * epoch becomes L; in epoch i > 1, S = (1 - loss_i / L) U_max.  Whole elements,
 * never negative (a loss above L means no stage 2), never above U_max.
 */
int64_t osp_oracle_tune_budget(int epoch, double loss_i, double L, double u_max,
                               int64_t model_elems)
{
    double limit = 0.8 * (double)model_elems;
    if (u_max > limit)
        u_max = limit;
    if (epoch == 1)
        return 0;
    double share = 1.0 - loss_i / L;
    if (share < 0.0)
        share = 0.0;
    if (share > 1.0)
        share = 1.0;
    return (int64_t)floor(share * u_max);
}
