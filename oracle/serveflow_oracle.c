/*
 * CPU oracle for the batched fast-slow flow classifier.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be checked
 * against a plain, slow, obviously-correct implementation.  It shares no code
 * with the GPU library, it is never called from the product path, and it is not
 * tuned for speed: every function below is the definition of the step written
 * out, one flow at a time.
 *
 * The method (fast model on every flow, an uncertainty gate, the slow model on
 * the uncertain subset only) is Section 3.1 and Section 3.2 of the paper.  The
 * paper does not fix a feature set, a tree storage format or a slow-model
 * architecture; where it is silent the readings below are used (each function
 * says which).
 *
 * Floating point: feature statistics are IEEE-754 binary32, every operation
 * rounded on its own (build with -ffp-contract=off, no fast-math).  The MLP
 * accumulates in binary64.
 *
 * Pins (tests/test_oracle_*.py): hand-computed statistics on dyadic inputs,
 * numpy's mean/std/min/max/median, a brute-force bit loop, hand-traced and
 * recursively walked trees, the multinomial closed form for the top-vote
 * histogram, set/ordering invariants of the gate, numpy's float64 matmul and
 * the identity / one-hot / dead-ReLU special cases of the MLP; for the tree tier
 * a decision tree fitted by scikit-learn (predict, predict_proba), a hand-traced
 * tree and exact rational arithmetic for the ratio gate; for the boosted form a
 * gradient-boosting classifier fitted by scikit-learn (decision_function,
 * predict_proba), scipy's softmax and entropy, and a sum whose result depends on
 * the order of the additions.
 * Accuracy of the classifier itself (F1 etc.) is parity unpinned: it needs the
 * paper's datasets and trained models.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_WINDOW 4096 /* packets of one flow the feature step looks at */

/* ------------------------------------------------------------------------- */
/* Step 1: features from the first k packets (context length k, Section 3.1).
 *
 * Reading used where the paper is silent:
 *   window w  = first m_w = min(n_i, depth[w]) packets of the flow, stored order;
 *   group g   = 0: packets with dir==0, 1: dir==1, 2: all packets of the window;
 *   quantity q= 0: packet size (as float), 1: stored inter-arrival time;
 *   five statistics s = mean, population std, min, max, median (mean of the
 *   two middle values for an even count); an empty group gives five zeros;
 *   column f = 32*w + 10*g + 5*q + s;  f = 32*w+30: total bytes;  32*w+31: m_w.
 */
static void stat5(const float *x, int c, float out[5])
{
    if (c == 0) {
        out[0] = out[1] = out[2] = out[3] = out[4] = 0.0f;
        return;
    }
    float sum = 0.0f;
    for (int j = 0; j < c; ++j)
        sum = sum + x[j];
    float mean = sum / (float)c;
    float ss = 0.0f;
    for (int j = 0; j < c; ++j) {
        float t = x[j] - mean;
        float t2 = t * t;
        ss = ss + t2;
    }
    float var = ss / (float)c;
    float sd = sqrtf(var);
    float mn = x[0], mx = x[0];
    for (int j = 1; j < c; ++j) {
        if (x[j] < mn) mn = x[j];
        if (x[j] > mx) mx = x[j];
    }
    /* ascending sort of a copy (insertion sort: c is tens of packets at most) */
    float s[ORACLE_MAX_WINDOW];
    for (int j = 0; j < c; ++j) {
        float v = x[j];
        int p = j;
        while (p > 0 && s[p - 1] > v) {
            s[p] = s[p - 1];
            --p;
        }
        s[p] = v;
    }
    float med;
    if (c & 1) {
        med = s[c / 2];
    } else {
        float two = s[c / 2 - 1] + s[c / 2];
        med = two * 0.5f;
    }
    out[0] = mean;
    out[1] = sd;
    out[2] = mn;
    out[3] = mx;
    out[4] = med;
}

static void featurize_flow(const uint16_t *size, const float *iat, const uint8_t *dir, uint32_t n,
                           uint32_t n_windows, const uint32_t *depth, float *f)
{
    float xs[ORACLE_MAX_WINDOW], xi[ORACLE_MAX_WINDOW];
    for (uint32_t w = 0; w < n_windows; ++w) {
        uint32_t m = n < depth[w] ? n : depth[w];
        float *fw = f + 32 * w;
        for (int g = 0; g < 3; ++g) {
            int c = 0;
            for (uint32_t j = 0; j < m; ++j) {
                if (g == 2 || dir[j] == (uint8_t)g) {
                    xs[c] = (float)size[j];
                    xi[c] = iat[j];
                    ++c;
                }
            }
            stat5(xs, c, fw + 10 * g);
            stat5(xi, c, fw + 10 * g + 5);
        }
        uint32_t bytes = 0;
        for (uint32_t j = 0; j < m; ++j)
            bytes += size[j];
        fw[30] = (float)bytes;
        fw[31] = (float)m;
    }
}

/* Raw header bits (the per-packet bit representation of Section 4.1): feature
 * r = raw_bits*j + b is bit b of packet j's header, bits numbered MSB-first in
 * each byte, header byte k stored in word k/4 at bit offset 8*(k%4).  Packets
 * past the end of the flow give zeros. */
static inline uint8_t header_bit(const uint32_t *words, uint32_t b)
{
    uint32_t k = b >> 3;
    uint32_t byte = (words[k >> 2] >> (8u * (k & 3u))) & 0xFFu;
    return (uint8_t)((byte >> (7u - (b & 7u))) & 1u);
}

/* returns 0 on success, -1 on invalid arguments */
int oracle_featurize(uint32_t n_flows, const uint32_t *flow_off, const uint16_t *pkt_size,
                     const float *pkt_iat, const uint8_t *pkt_dir, const uint32_t *pkt_hdr,
                     uint32_t hdr_words, uint32_t n_windows, const uint32_t *depth,
                     uint32_t raw_pkts, uint32_t raw_bits, float *feat, uint32_t feat_ld,
                     uint8_t *raw, int n_threads)
{
    if (n_windows < 1 || feat_ld < 32 * n_windows) return -1;
    for (uint32_t w = 0; w < n_windows; ++w) {
        if (depth[w] < 1 || depth[w] > ORACLE_MAX_WINDOW) return -1;
        if (w && depth[w] <= depth[w - 1]) return -1;
    }
    if (raw && (!pkt_hdr || raw_bits > 32 * hdr_words)) return -1;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int64_t i = 0; i < (int64_t)n_flows; ++i) {
        uint32_t o = flow_off[i], n = flow_off[i + 1] - flow_off[i];
        featurize_flow(pkt_size + o, pkt_iat + o, pkt_dir + o, n, n_windows, depth,
                       feat + (size_t)i * feat_ld);
        if (raw) {
            uint8_t *r = raw + (size_t)i * raw_pkts * raw_bits;
            for (uint32_t j = 0; j < raw_pkts; ++j)
                for (uint32_t b = 0; b < raw_bits; ++b)
                    r[(size_t)j * raw_bits + b] =
                        j < n ? header_bit(pkt_hdr + (size_t)(o + j) * hdr_words, b) : 0;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Steps 2-3: the fast model sees every flow (Section 3.1).  Here it is a hard-
 * voting ensemble of perfect binary trees of depth d in heap order: from node k
 * go to 2k+1 if x[feat[k]] <= thr[k], else to 2k+2; after d steps the leaf is
 * k - (2^d - 1).  votes[c] counts trees whose leaf is labelled c.  With
 * P(y|x) = votes[y]/T the least-confidence score of Section 3.2 is
 * LC = 1 - top_votes/T, so the integer top_votes carries the score exactly.
 * Ties in the arg-max go to the lowest class index. */
int oracle_fast_infer(uint32_t n_flows, const float *feat, uint32_t feat_ld, uint32_t n_trees,
                      uint32_t depth, uint32_t n_classes, uint32_t n_features,
                      const uint16_t *node_feat, const float *node_thr, const uint8_t *leaf_label,
                      uint16_t *votes, uint16_t *pred, uint16_t *top_votes, uint16_t *leaf_idx,
                      int n_threads)
{
    if (depth < 1 || depth > 16 || n_classes < 1 || n_classes > 65535 || n_features > feat_ld) return -1;
    const uint32_t n_int = (1u << depth) - 1u, n_leaf = 1u << depth;
    for (size_t q = 0; q < (size_t)n_trees * n_int; ++q)
        if (node_feat[q] >= n_features) return -1;
    for (size_t q = 0; q < (size_t)n_trees * n_leaf; ++q)
        if (leaf_label[q] >= n_classes) return -1;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int64_t i = 0; i < (int64_t)n_flows; ++i) {
        const float *x = feat + (size_t)i * feat_ld;
        uint32_t *v = (uint32_t *)calloc(n_classes, sizeof(uint32_t));
        for (uint32_t t = 0; t < n_trees; ++t) {
            const uint16_t *nf = node_feat + (size_t)t * n_int;
            const float *nt = node_thr + (size_t)t * n_int;
            uint32_t k = 0;
            for (uint32_t s = 0; s < depth; ++s)
                k = 2 * k + 1 + (x[nf[k]] <= nt[k] ? 0u : 1u);
            uint32_t leaf = k - n_int;
            if (leaf_idx) leaf_idx[(size_t)i * n_trees + t] = (uint16_t)leaf;
            v[leaf_label[(size_t)t * n_leaf + leaf]] += 1;
        }
        uint32_t best = 0;
        for (uint32_t c = 1; c < n_classes; ++c)
            if (v[c] > v[best]) best = c;
        pred[i] = (uint16_t)best;
        top_votes[i] = (uint16_t)v[best];
        if (votes)
            for (uint32_t c = 0; c < n_classes; ++c)
                votes[(size_t)i * n_classes + c] = (uint16_t)v[c];
        free(v);
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Step 4: the gate.  "Vote fraction below theta" is evaluated in integers:
 * vmin = ceil(theta*T), formed exactly (a 24-bit significand times T < 2^16 fits
 * a double), and a flow escalates iff top_votes < vmin.  Equivalent to
 * LC(x) > 1 - theta of Section 3.2 without rounding the fraction. */
uint32_t oracle_vmin_from_theta(float theta, uint32_t n_trees)
{
    double p = (double)theta * (double)n_trees;
    double c = ceil(p);
    if (c < 0.0) c = 0.0;
    if (c > 65535.0) c = 65535.0;
    return (uint32_t)c;
}

/* n_vmin == 1: one threshold for all flows (universal form, Section 3.2);
 * n_vmin == n_classes: vmin[pred] (per-class form).  The list is ascending in
 * flow index.  Returns the number of escalated flows. */
uint32_t oracle_route(uint32_t n_flows, const uint16_t *top_votes, const uint16_t *pred,
                      const uint16_t *vmin, uint32_t n_vmin, uint32_t *esc_idx)
{
    uint32_t e = 0;
    for (uint32_t i = 0; i < n_flows; ++i) {
        uint16_t th = n_vmin == 1 ? vmin[0] : vmin[pred[i]];
        if (top_votes[i] < th) esc_idx[e++] = i;
    }
    return e;
}

/* ------------------------------------------------------------------------- */
/* The tier in front of the fast model (Section 3.1: the "fastest" model, a single
 * decision tree, sees every flow first; Section 4.1: its leaves keep enough
 * training samples, at least 15, for the leaf's class distribution to serve as the
 * uncertainty estimate).
 *
 * Reading used where the paper is silent: a perfect binary tree in heap order with
 * the same split rule as the forest (x[f] <= thr goes left); leaf_count[leaf][c]
 * = number of training samples of class c that reached the leaf;
 *   P(y|x) = leaf_count[leaf][y] / leaf_total,  leaf_total = sum_c leaf_count[leaf][c];
 *   pred = arg-max, lowest class on ties;  top_count = leaf_count[leaf][pred];
 *   LC(x) = 1 - top_count / leaf_total  (Section 3.2).
 * A leaf total must fit 16 bits. */
int oracle_tree_infer(uint32_t n_flows, const float *feat, uint32_t feat_ld, uint32_t depth,
                      uint32_t n_classes, uint32_t n_features, const uint16_t *node_feat,
                      const float *node_thr, const uint16_t *leaf_count /* [2^depth][n_classes] */,
                      uint16_t *pred, uint16_t *top_count, uint16_t *leaf_total,
                      uint16_t *leaf_idx /* [n_flows] or NULL */, int n_threads)
{
    if (depth < 1 || depth > 15 || n_classes < 1 || n_features < 1 || n_features > feat_ld) return -1;
    const uint32_t n_int = (1u << depth) - 1u, n_leaf = 1u << depth;
    for (uint32_t q = 0; q < n_int; ++q)
        if (node_feat[q] >= n_features) return -1;
    for (uint32_t l = 0; l < n_leaf; ++l) {
        uint64_t tot = 0;
        for (uint32_t c = 0; c < n_classes; ++c) tot += leaf_count[(size_t)l * n_classes + c];
        if (tot > 65535u) return -1;
    }
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int64_t i = 0; i < (int64_t)n_flows; ++i) {
        const float *x = feat + (size_t)i * feat_ld;
        uint32_t k = 0;
        for (uint32_t s = 0; s < depth; ++s)
            k = 2 * k + 1 + (x[node_feat[k]] <= node_thr[k] ? 0u : 1u);
        const uint32_t leaf = k - n_int;
        const uint16_t *cnt = leaf_count + (size_t)leaf * n_classes;
        uint32_t best = 0, tot = 0;
        for (uint32_t c = 0; c < n_classes; ++c) {
            tot += cnt[c];
            if (cnt[c] > cnt[best]) best = c;
        }
        pred[i] = (uint16_t)best;
        top_count[i] = cnt[best];
        leaf_total[i] = (uint16_t)tot;
        if (leaf_idx) leaf_idx[i] = (uint16_t)leaf;
    }
    return 0;
}

/* top/total < theta without rounding anything: theta = m * 2^e with an integer m
 * (a binary32 value has 24 significant bits), so the test is top * 2^-e < m * total
 * in integers.  A leaf without samples has no distribution: P(y|x) is read as 0 for
 * every y, LC = 1, and the flow escalates for any positive theta. */
static int ratio_below(uint32_t top, uint32_t total, float theta)
{
    if (!(theta > 0.0f)) return 0;
    if (total == 0) return 1;
    int e;
    double fr = frexp((double)theta, &e);          /* theta = fr * 2^e, 0.5 <= fr < 1 */
    unsigned __int128 m = (unsigned __int128)(uint64_t)ldexp(fr, 24);
    e -= 24;                                       /* theta = m * 2^e, m < 2^24       */
    unsigned __int128 lhs = top, rhs = m * total;  /* rhs < 2^40                      */
    if (e >= 0) {
        if (e > 64) return 1;                      /* theta*total >= 2^64 > top       */
        rhs <<= e;
    } else {
        if (-e > 64) return top == 0;              /* theta*total < 1                 */
        lhs <<= -e;
    }
    return lhs < rhs;
}

/* Gate of the tree tier: escalate iff max_y P(y|x) < theta, i.e. LC(x) > 1 - theta
 * (Section 3.2).  Ascending index list; returns its length. */
uint32_t oracle_route_ratio(uint32_t n_flows, const uint16_t *top_count, const uint16_t *leaf_total,
                            float theta, uint32_t *esc_idx)
{
    uint32_t e = 0;
    for (uint32_t i = 0; i < n_flows; ++i)
        if (ratio_below(top_count[i], leaf_total[i], theta)) esc_idx[e++] = i;
    return e;
}

/* ------------------------------------------------------------------------- */
/* Boosted-tree form of the fast model (Section 4.1 names gradient-boosted trees,
 * the fast and slow models of the evaluated cascade in Section 5.2 are of that
 * kind) with the two uncertainty scores of Section 3.2:
 *   LC(x) = 1 - max_y P(y|x)          H(x) = - sum_i P(y_i|x) log P(y_i|x).
 *
 * Reading used where the paper is silent (the usual multiclass boosting layout):
 * tree t belongs to class t mod C and boosting round t div C; its leaves hold a
 * binary32 margin; the class margin is
 *   m[c] = base[c] + leaf(c) + leaf(C + c) + leaf(2C + c) + ...
 * added in that order, every addition rounded to binary32 (so that a second
 * implementation can reproduce it bit for bit);  P(.|x) = softmax(m), evaluated
 * in binary64 from the binary32 margins with the maximum subtracted first;
 * pred = arg-max of m, lowest class on ties; log is natural; 0 log 0 = 0.
 * Trees are perfect, heap order, x[f] <= thr goes left, as everywhere here. */
int oracle_gbdt_infer(uint32_t n_flows, const float *feat, uint32_t feat_ld, uint32_t n_trees,
                      uint32_t depth, uint32_t n_classes, uint32_t n_features,
                      const uint16_t *node_feat, const float *node_thr,
                      const float *leaf_value /* [n_trees][2^depth] */, const float *base /* [C] */,
                      float *margin /* [n][C] or NULL */, uint16_t *pred, double *lc, double *entropy,
                      int n_threads)
{
    if (depth < 1 || depth > 15 || n_classes < 1 || n_trees < 1 || n_features > feat_ld) return -1;
    const uint32_t n_int = (1u << depth) - 1u, n_leaf = 1u << depth;
    for (size_t q = 0; q < (size_t)n_trees * n_int; ++q)
        if (node_feat[q] >= n_features) return -1;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int64_t i = 0; i < (int64_t)n_flows; ++i) {
        const float *x = feat + (size_t)i * feat_ld;
        float *m = (float *)malloc(sizeof(float) * n_classes);
        for (uint32_t c = 0; c < n_classes; ++c) m[c] = base ? base[c] : 0.0f;
        for (uint32_t t = 0; t < n_trees; ++t) {
            const uint16_t *nf = node_feat + (size_t)t * n_int;
            const float *nt = node_thr + (size_t)t * n_int;
            uint32_t k = 0;
            for (uint32_t s = 0; s < depth; ++s)
                k = 2 * k + 1 + (x[nf[k]] <= nt[k] ? 0u : 1u);
            float v = leaf_value[(size_t)t * n_leaf + (k - n_int)];
            m[t % n_classes] = m[t % n_classes] + v;
        }
        uint32_t best = 0;
        for (uint32_t c = 1; c < n_classes; ++c)
            if (m[c] > m[best]) best = c;
        double z = 0.0;
        for (uint32_t c = 0; c < n_classes; ++c) z += exp((double)m[c] - (double)m[best]);
        double h = 0.0;
        for (uint32_t c = 0; c < n_classes; ++c) {
            double p = exp((double)m[c] - (double)m[best]) / z;
            if (p > 0.0) h -= p * log(p);
        }
        pred[i] = (uint16_t)best;
        lc[i] = 1.0 - 1.0 / z; /* the largest probability is exp(0) / z */
        entropy[i] = h;
        if (margin)
            for (uint32_t c = 0; c < n_classes; ++c) margin[(size_t)i * n_classes + c] = m[c];
        free(m);
    }
    return 0;
}

/* Gate on a real-valued uncertainty score (Section 3.2): a flow is assigned to the
 * slower model iff its score exceeds the threshold.  Ascending list; returns its length. */
uint32_t oracle_route_score(uint32_t n_flows, const float *score, float threshold, uint32_t *esc_idx)
{
    uint32_t e = 0;
    for (uint32_t i = 0; i < n_flows; ++i)
        if (score[i] > threshold) esc_idx[e++] = i;
    return e;
}

/* Universal uncertainty thresholds (Algorithm 1): sort the scores ascending and
 * read, for each quantile q, the element at 1-based position ceil(q*|U|)
 * (1-based because the position can equal |U|; position 0 is read as 1). */
static int cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}
int oracle_universal_thresholds(const double *scores, uint32_t n, const double *q, uint32_t nq,
                                double *thresholds)
{
    if (n == 0) return -1;
    double *u = (double *)malloc(sizeof(double) * n);
    memcpy(u, scores, sizeof(double) * n);
    qsort(u, n, sizeof(double), cmp_double);
    for (uint32_t j = 0; j < nq; ++j) {
        double pos = ceil(q[j] * (double)n);
        if (pos < 1.0) pos = 1.0;
        if (pos > (double)n) pos = (double)n;
        thresholds[j] = u[(uint32_t)pos - 1];
    }
    free(u);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Step 5: the slow model runs on escalated flows only and its answer replaces
 * the fast one (Sections 3.1, 4.4).  Here it is a 3-layer ReLU MLP.
 *   input map   z_f = clamp((x_f - mu_f) * inv_sigma_f, -c, +c) in binary32, one
 *               rounding per operation; identity when mu is NULL; for a bf16 model
 *               z is then rounded to bfloat16 (ties to even);
 *   layers      binary64 products and sums, ReLU(v) = max(v, 0), hidden values
 *               kept unrounded; logits rounded to binary32 at the end;
 *   label       arg-max, lowest index on ties; written to labels[flow].
 * Weights are row-major [out][in] float arrays (already bf16-representable for a
 * bf16 model). */
static float bf16_round(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return x; /* inf/nan unchanged */
    u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
    memcpy(&x, &u, 4);
    return x;
}

int oracle_slow_infer(uint32_t n_esc, const uint32_t *esc_idx,
                      const float *feat, uint32_t feat_ld,                 /* stat-feature input, or */
                      const uint32_t *flow_off, const uint32_t *pkt_hdr,   /* raw-bit input          */
                      uint32_t hdr_words, uint32_t raw_pkts, uint32_t raw_bits,
                      uint32_t n_in, uint32_t n_h1, uint32_t n_h2, uint32_t n_classes, int is_bf16,
                      const float *mu, const float *inv_sigma, float clamp,
                      const float *w1, const float *b1, const float *w2, const float *b2,
                      const float *w3, const float *b3,
                      float *logits /* [n_esc][n_classes] */, uint16_t *labels /* [n_flows] */,
                      int n_threads)
{
    const int raw_mode = feat == NULL;
    if (raw_mode && (!flow_off || !pkt_hdr || raw_pkts * raw_bits != n_in)) return -1;
    if (!raw_mode && n_in > feat_ld) return -1;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int64_t e = 0; e < (int64_t)n_esc; ++e) {
        uint32_t i = esc_idx[e];
        double *z = (double *)malloc(sizeof(double) * ((size_t)n_in + n_h1 + n_h2));
        double *h1 = z + n_in, *h2 = h1 + n_h1;
        if (raw_mode) {
            uint32_t o = flow_off[i], n = flow_off[i + 1] - flow_off[i];
            for (uint32_t j = 0; j < raw_pkts; ++j)
                for (uint32_t b = 0; b < raw_bits; ++b)
                    z[(size_t)j * raw_bits + b] =
                        j < n ? (double)header_bit(pkt_hdr + (size_t)(o + j) * hdr_words, b) : 0.0;
        } else {
            const float *x = feat + (size_t)i * feat_ld;
            for (uint32_t f = 0; f < n_in; ++f) {
                float v = x[f];
                if (mu) {
                    float d = v - mu[f];
                    v = d * inv_sigma[f];
                    if (v < -clamp) v = -clamp;
                    if (v > clamp) v = clamp;
                }
                if (is_bf16) v = bf16_round(v);
                z[f] = (double)v;
            }
        }
        for (uint32_t o = 0; o < n_h1; ++o) {
            double acc = 0.0;
            for (uint32_t f = 0; f < n_in; ++f)
                acc += (double)w1[(size_t)o * n_in + f] * z[f];
            acc += (double)b1[o];
            h1[o] = acc > 0.0 ? acc : 0.0;
        }
        for (uint32_t o = 0; o < n_h2; ++o) {
            double acc = 0.0;
            for (uint32_t f = 0; f < n_h1; ++f)
                acc += (double)w2[(size_t)o * n_h1 + f] * h1[f];
            acc += (double)b2[o];
            h2[o] = acc > 0.0 ? acc : 0.0;
        }
        uint32_t best = 0;
        float best_v = 0.0f;
        for (uint32_t o = 0; o < n_classes; ++o) {
            double acc = 0.0;
            for (uint32_t f = 0; f < n_h2; ++f)
                acc += (double)w3[(size_t)o * n_h2 + f] * h2[f];
            acc += (double)b3[o];
            float lv = (float)acc;
            if (logits) logits[(size_t)e * n_classes + o] = lv;
            if (o == 0 || lv > best_v) {
                best = o;
                best_v = lv;
            }
        }
        if (labels) labels[i] = (uint16_t)best;
        free(z);
    }
    return 0;
}

int oracle_max_window(void) { return ORACLE_MAX_WINDOW; }
