/*
 * serveflow.h - C ABI of the batched fast-slow flow classifier for AMD MI355X (gfx950).
 *
 * The library runs the data-parallel hot path of a fast-slow model architecture for
 * network traffic analysis (Section 3.1 of the paper): every flow is featurised from its
 * first k packets and classified by a fast tree ensemble; an uncertainty score decides
 * which flows are certain enough (Section 3.2); the uncertain ones are compacted into a
 * list and re-classified by a slower dense model, whose label replaces the fast one.
 * Around these four steps: a decision tree as a tier in front (the three-tier cascade of
 * Section 3.1), gradient-boosted trees as the fast model with the entropy score, the threshold
 * algorithms of Section 3.2, and the flow-ID join of the two queues in front of the slow model.
 *
 * Conventions that hold for every entry point
 *   - Pointers inside the structs and pointer arguments are DEVICE pointers unless the
 *     name starts with host_.  The structs themselves live in host memory.
 *   - The caller owns every buffer.  The library owns only the sf_ctx object.  No entry
 *     point allocates or frees device memory; scratch comes from the workspace handed to
 *     sf_create.
 *   - Work is enqueued on the context's HIP stream and the call returns without waiting;
 *     outputs are valid once the caller has synchronised that stream.  (sf_validate_* are
 *     the exception: they wait and report.)
 *   - Every call returns an int status (SF_OK = 0, negative = error), never throws and
 *     never aborts.  Argument errors that the host can see return SF_EINVAL before
 *     anything is launched; sf_last_error() then describes the problem.
 *   - Kernels clamp offsets and indices read from device memory into range, so malformed
 *     device data gives wrong answers, not memory faults; sf_validate_* finds such data.
 *   - Calls on one context must not overlap (one stream, one workspace).
 */
#ifndef SERVEFLOW_H
#define SERVEFLOW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sf_ctx sf_ctx;

enum {
    SF_OK = 0,
    SF_EINVAL = -1,       /* bad argument (null pointer, size out of range, bad layout)   */
    SF_ENOMEM = -2,       /* workspace too small for this call                           */
    SF_EHIP = -3,         /* a HIP runtime call failed; see sf_last_error                */
    SF_EUNSUPPORTED = -4, /* a size beyond the compiled limits                           */
    SF_EDATA = -5         /* sf_validate_*: device data violates the documented layout   */
};

enum { SF_F32 = 0, SF_BF16 = 1 };

/* compiled limits */
#define SF_MAX_WINDOWS 4     /* prefix windows per flow                                  */
#define SF_MAX_DEPTH_PKTS 64 /* packets of a flow the feature step looks at              */
#define SF_MAX_FEATURES 128  /* 32 * SF_MAX_WINDOWS                                      */
#define SF_MAX_TREE_DEPTH 14
#define SF_MAX_CLASSES 64
#define SF_HDR_WORDS_MAX 32  /* 1024 header bits per packet                              */

/* ---- context ------------------------------------------------------------------------ */

/* Scratch bytes that cover every entry point for at most max_flows flows per call, a
 * forest of n_trees trees of depth tree_depth and an MLP n_in -> n_h1 -> n_h2 -> classes
 * (pass zeros for the parts not used).  Host function, no GPU needed. */
size_t sf_workspace_bytes(uint32_t max_flows, uint32_t n_trees, uint32_t tree_depth,
                          uint32_t n_in, uint32_t n_h1, uint32_t n_h2);

/* Create a context bound to hip_stream (a hipStream_t; NULL = the default stream) and to
 * a caller-owned device workspace of workspace_bytes bytes (256-byte aligned).  The
 * workspace must stay valid until sf_destroy.  Needs a GPU. */
int sf_create(sf_ctx** out, void* hip_stream, void* workspace, size_t workspace_bytes);
void sf_destroy(sf_ctx* ctx);
/* Text of the last error on this context (or of the last failed sf_create when ctx is
 * NULL).  The string belongs to the library; it stays valid until the next call. */
const char* sf_last_error(const sf_ctx* ctx);

/* ---- step 1: features from the first k packets ---------------------------------------
 * Section 3.1: the amount of context (first k packets) is the key parameter; packet sizes,
 * inter-arrival times and direction are the flow-level inputs; Section 4.1: the raw header
 * bits of each packet are the alternative representation.
 *
 * Packet records are SoA, grouped by flow (CSR): flow i owns packets
 * [flow_off[i], flow_off[i+1]).  For window w the first m = min(n_i, depth[w]) packets are
 * summarised as 32 floats: for group g in (dir==0, dir==1, all) and quantity q in (size,
 * inter-arrival time) the five statistics mean, population std, min, max, median, at column
 * 32*w + 10*g + 5*q + s; column 32*w+30 = total bytes, 32*w+31 = m.  An empty group gives
 * zeros.  All arithmetic is binary32, one rounding per operation, sums in packet order,
 * variance by the two-pass formula. */
typedef struct {
    uint32_t n_flows;
    uint64_t n_pkts;
    const uint32_t* flow_off; /* [n_flows+1], flow_off[0] = 0, non-decreasing, last = n_pkts */
    const uint16_t* pkt_size; /* [n_pkts] bytes                                              */
    const float* pkt_iat;     /* [n_pkts] seconds, finite                                    */
    const uint8_t* pkt_dir;   /* [n_pkts] 0 or 1                                             */
    const uint32_t* pkt_hdr;  /* optional [n_pkts][hdr_words]: header byte k is bits
                                 8*(k%4)..8*(k%4)+7 of word k/4; header bit b is bit 7-(b%8)
                                 of byte b/8.  May be NULL.                                   */
    uint32_t hdr_words;       /* words per packet in pkt_hdr (15 for 480 bits), 0 if NULL     */
} sf_packets;

typedef struct {
    uint32_t n_windows;               /* 1..SF_MAX_WINDOWS                                  */
    uint32_t depth[SF_MAX_WINDOWS];   /* strictly increasing, 1..SF_MAX_DEPTH_PKTS          */
    uint32_t raw_pkts, raw_bits;      /* raw header-bit features: first raw_pkts packets x
                                         raw_bits bits each (0,0 = none)                    */
} sf_feat_cfg;

/* feat: [n_flows][feat_ld] float, feat_ld >= 32*n_windows; columns beyond 32*n_windows are
 * left untouched.  raw: optional [n_flows][raw_pkts*raw_bits] bytes in {0,1} (feature
 * raw_bits*j + b = header bit b of packet j, zeros past the end of the flow); NULL skips it.
 * n_flows = 0 is a successful no-op. */
int sf_featurize(sf_ctx* ctx, const sf_packets* pk, const sf_feat_cfg* cfg, float* feat,
                 uint32_t feat_ld, uint8_t* raw);

/* Waits for the stream, then checks the CSR layout on the device: flow_off[0] = 0,
 * non-decreasing, last = n_pkts, pkt_dir in {0,1}, pkt_iat finite.  SF_EDATA if violated. */
int sf_validate_packets(sf_ctx* ctx, const sf_packets* pk);

/* ---- steps 2-3: fast model on every flow, uncertainty score ---------------------------
 * Section 3.1: the fast model sees all traffic.  Section 3.2: least confidence
 * LC(x) = 1 - max_y P(y|x).  The fast model here is a hard-voting ensemble of perfect
 * binary trees; with P(y|x) = votes[y] / n_trees the score is carried exactly by the
 * integer top_votes = max_y votes[y] (LC = 1 - top_votes / n_trees).
 *
 * Trees are stored in heap order: node k of tree t tests x[node_feat[t][k]] <= node_thr[t][k];
 * true goes to 2k+1, false to 2k+2; after depth steps the leaf is k - (2^depth - 1) and the
 * tree votes leaf_label[t][leaf].  pred = the class with most votes, lowest index on ties. */
typedef struct {
    uint32_t n_trees, depth, n_classes, n_features; /* depth 1..SF_MAX_TREE_DEPTH           */
    const uint16_t* node_feat; /* [n_trees][2^depth - 1], values < n_features               */
    const float* node_thr;     /* [n_trees][2^depth - 1]                                    */
    const uint8_t* leaf_label; /* [n_trees][2^depth], values < n_classes                    */
    const void* packed;        /* optional: what sf_forest_pack wrote for these node arrays;
                                  NULL = the nodes are re-packed into the workspace per call */
} sf_forest;

/* The kernels walk a packed copy of node_feat / node_thr.  A caller that keeps a model across
 * calls can have it made once: sf_forest_pack writes sf_forest_packed_bytes(n_trees, depth)
 * bytes to packed (device, 256-byte aligned, caller-owned) on the context's stream; set
 * forest->packed to it afterwards (and leave the node arrays unchanged while it is in use). */
size_t sf_forest_packed_bytes(uint32_t n_trees, uint32_t depth);
int sf_forest_pack(sf_ctx* ctx, const sf_forest* forest, void* packed);

/* feat: [n_flows][feat_ld], n_features <= feat_ld.  pred, top_votes: [n_flows].
 * votes: optional [n_flows][n_classes]; leaf_idx: optional [n_flows][n_trees] (for parity
 * checks).  Uses workspace for a packed copy of the forest (sf_forest_packed_bytes) unless
 * forest->packed is set. */
int sf_fast_infer(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_flows,
                  const sf_forest* forest, uint16_t* votes, uint16_t* pred,
                  uint16_t* top_votes, uint16_t* leaf_idx);

/* Waits, then checks node_feat < n_features and leaf_label < n_classes on the device. */
int sf_validate_forest(sf_ctx* ctx, const sf_forest* forest);

/* ---- step 4: the gate ------------------------------------------------------------------
 * Section 3.2: flows whose uncertainty exceeds a threshold are assigned to the slower model.
 * In integers: flow i escalates iff top_votes[i] < vmin, with vmin = ceil(theta * n_trees)
 * for "vote fraction below theta" (sf_vmin_from_theta forms it exactly).  host_vmin holds
 * one threshold (n_vmin = 1, universal) or one per class (n_vmin = number of classes,
 * threshold = host_vmin[pred[i]]; pred values >= n_vmin use the last entry).
 * esc_idx receives the escalated flow indices in ascending order (capacity n_flows),
 * *esc_count their number; both stay on the device. */
int sf_route(sf_ctx* ctx, const uint16_t* top_votes, const uint16_t* pred, uint32_t n_flows,
             const uint16_t* host_vmin, uint32_t n_vmin, uint32_t* esc_idx,
             uint32_t* esc_count);

/* sf_route for callers that cannot allocate device memory or hand over a workspace for this step
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, same results, but the per-block counts between its two launches live in a 16 KB array
 * that is part of the library's device code (one copy per GPU, held until the process ends) instead
 * of the context's workspace.  The call allocates nothing, on the host or on the device.
 * At most SF_ROUTE_STATIC_MAX_FLOWS flows per call (SF_EUNSUPPORTED beyond).  Every call on a GPU
 * uses that GPU's one array, whatever the context or stream: calls that overlap on one GPU race
 * (calls in stream order are fine; nothing in the array has to be cleared between them). */
#define SF_ROUTE_STATIC_MAX_FLOWS 2147483648u
int sf_route_static(sf_ctx* ctx, const uint16_t* top_votes, const uint16_t* pred, uint32_t n_flows,
                    const uint16_t* host_vmin, uint32_t n_vmin, uint32_t* esc_idx, uint32_t* esc_count);

/* ceil(theta * n_trees), exact for theta's binary32 value, clamped to 0..65535.  Host. */
uint32_t sf_vmin_from_theta(float theta, uint32_t n_trees);

/* ---- threshold calibration (Section 3.2, Algorithm 1 and "Determining the optimal threshold") ----
 * The uncertainty score here takes only n_trees+1 values, so its sorted list is a histogram.
 *
 * sf_score_histogram: host_hist[v] (v = 0..n_trees, n_trees+1 words, HOST memory) = number of flows
 * with top_votes == v (device array, [n_flows]).  Runs on the device, then waits for the stream. */
int sf_score_histogram(sf_ctx* ctx, const uint16_t* top_votes, uint32_t n_flows, uint32_t n_trees,
                       uint32_t* host_hist);

/* Algorithm 1 (universal uncertainty thresholds) on that histogram: sort the scores
 * LC = 1 - top_votes/n_trees ascending and, for each quantile q, take the element at 1-based
 * position ceil(q * n) (position 0 is read as 1).  host_votes_at[j] receives the top_votes value v
 * of that element, i.e. the threshold is LC = 1 - v/n_trees; escalating the flows with LC above it
 * is the gate vmin = v, which assigns at most a fraction 1 - q of the flows.  Host function. */
int sf_universal_thresholds(const uint32_t* host_hist, uint32_t n_trees, const double* host_q, uint32_t n_q,
                            uint16_t* host_votes_at);

/* The "target portion" way of fixing the threshold: the vmin (0..n_trees+1) whose escalated
 * fraction (flows with top_votes < vmin) is nearest target_fraction; on a tie the smaller fraction.
 * *reached_fraction (optional) receives the fraction actually reached.  Host function. */
uint32_t sf_vmin_for_target(const uint32_t* host_hist, uint32_t n_trees, double target_fraction,
                            double* reached_fraction);

/* Slope-based per-class thresholds (Section 3.2, Algorithm 2), for a validation set whose true labels
 * are known.  sf_class_score_histogram: host_hist[((c * (n_trees+1)) + v) * 2 + w] (HOST memory,
 * n_classes * (n_trees+1) * 2 words) = number of flows with pred == c, top_votes == v and w = 0 for a
 * correct prediction (pred == truth), 1 for an incorrect one; top_votes, pred, truth are device arrays
 * of n_flows entries.  Runs on the device, then waits for the stream.
 *
 * sf_per_class_thresholds (host function): every class starts with nothing assigned; a class's
 * candidates are its non-empty vote counts, fewest votes (highest uncertainty) first; a candidate
 * assigns dC correct and dI incorrect flows and has slope dI / (dC + dI); each increment takes the
 * steepest next candidate over the classes (exact comparison; lowest class on ties) until the
 * assigned total reaches target_fraction of the flows or nothing is left.  host_vmin[c] receives the
 * class's threshold for sf_route's per-class form (flow escalates iff top_votes < host_vmin[pred]);
 * *reached_fraction (optional) the assigned fraction. */
int sf_class_score_histogram(sf_ctx* ctx, const uint16_t* top_votes, const uint16_t* pred, const uint16_t* truth,
                             uint32_t n_flows, uint32_t n_trees, uint32_t n_classes, uint32_t* host_hist);
int sf_per_class_thresholds(const uint32_t* host_hist, uint32_t n_trees, uint32_t n_classes, double target_fraction,
                            uint16_t* host_vmin, double* reached_fraction);

/* ---- three tiers: a single decision tree in front of the fast model ----------------------
 * Section 3.1: a "fastest" model (a decision tree) sees every flow first; only the flows it
 * is unsure of go on to the fast model, and only those the fast model is unsure of reach the
 * slow one.  Section 4.1: the tree's leaves keep the class counts of their training samples
 * (at least 15 per leaf), which make the leaf a distribution: P(y|x) = leaf_count[leaf][y] /
 * leaf_total, leaf_total = sum over y.  Section 3.2: LC(x) = 1 - max_y P(y|x).
 *
 * The tree is perfect, in heap order, with the split rule of sf_forest.  pred = the class
 * with the largest count at the leaf (lowest index on ties), top_count = that count. */
typedef struct {
    uint32_t depth, n_classes, n_features; /* depth 1..SF_MAX_TREE_DEPTH                      */
    const uint16_t* node_feat;  /* [2^depth - 1], values < n_features                          */
    const float* node_thr;      /* [2^depth - 1]                                               */
    const uint16_t* leaf_count; /* [2^depth][n_classes]; a leaf's counts sum to at most 65535  */
} sf_tree;

/* feat: [n_flows][feat_ld].  pred, top_count, leaf_total: [n_flows]; leaf_idx: optional
 * [n_flows] (for parity checks).  Uses workspace (16 bytes per leaf). */
int sf_fastest_infer(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_flows,
                     const sf_tree* tree, uint16_t* pred, uint16_t* top_count, uint16_t* leaf_total,
                     uint16_t* leaf_idx);

/* Waits, then checks node_feat < n_features, leaf totals <= 65535 and thresholds not NaN. */
int sf_validate_tree(sf_ctx* ctx, const sf_tree* tree);

/* The gate of the tree tier: flow i escalates iff top_count[i] / leaf_total[i] < theta, i.e.
 * LC above 1 - theta, evaluated without rounding (theta's binary32 value times a 16-bit total
 * is exact in binary64).  A leaf without samples (leaf_total 0) escalates for any theta > 0.
 * Outputs as sf_route. */
int sf_route_ratio(sf_ctx* ctx, const uint16_t* top_count, const uint16_t* leaf_total, uint32_t n_flows,
                   float theta, uint32_t* esc_idx, uint32_t* esc_count);

/* The fast model on the flows of a list only.  idx / idx_count: as written by sf_route or
 * sf_route_ratio (device); at most idx_cap entries are read; entries >= n_flows are clamped.
 * Row j of the outputs belongs to flow idx[j]: pred, top_votes: [idx_cap]; votes: optional
 * [idx_cap][n_classes].  labels: optional [n_flows]; labels[idx[j]] = pred[j] (the fast
 * label replaces the tree's).  Rows from *idx_count on are not written. */
int sf_fast_infer_subset(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_flows,
                         const uint32_t* idx, const uint32_t* idx_count, uint32_t idx_cap,
                         const sf_forest* forest, uint16_t* votes, uint16_t* pred, uint16_t* top_votes,
                         uint16_t* labels);

/* sf_route over the rows of such a list: row j escalates iff top_votes[j] < vmin (per-class:
 * host_vmin[pred[j]]); esc_idx receives the FLOW numbers idx[j] of the escalated rows, which
 * are ascending because idx is; *esc_count their number.  Capacity of esc_idx: idx_cap. */
int sf_route_subset(sf_ctx* ctx, const uint16_t* top_votes, const uint16_t* pred, const uint32_t* idx,
                    const uint32_t* idx_count, uint32_t idx_cap, const uint16_t* host_vmin, uint32_t n_vmin,
                    uint32_t* esc_idx, uint32_t* esc_count);

/* ---- boosted trees as the fast model, real-valued uncertainty scores ----------------------
 * Section 4.1 names gradient-boosted trees among the models (the fast and slow models of the
 * cascade evaluated in Section 5.2 are of that kind); Section 3.2 gives two scores on the
 * model's class distribution: least confidence LC(x) = 1 - max_y P(y|x) and entropy
 * H(x) = - sum_i P(y_i|x) log P(y_i|x).
 *
 * Tree t belongs to class t mod n_classes (boosting round t div n_classes); its leaves hold
 * binary32 margins.  m[c] = base[c] + the leaf values of the class's trees, added in tree
 * order, each addition rounded to binary32 (reproducible bit for bit).  P = softmax(m),
 * evaluated in binary64; pred = arg-max of m, lowest class on ties; natural logarithm.
 * Trees: perfect, heap order, x[f] <= thr goes left (as sf_forest). */
typedef struct {
    uint32_t n_trees, depth, n_classes, n_features;
    const uint16_t* node_feat; /* [n_trees][2^depth - 1], values < n_features                  */
    const float* node_thr;     /* [n_trees][2^depth - 1]                                       */
    const float* leaf_value;   /* [n_trees][2^depth]                                           */
    const float* base;         /* [n_classes] initial margins, or NULL for zeros               */
    const void* packed;        /* optional, as in sf_forest (sf_gbdt_pack, same size formula)  */
} sf_gbdt;

int sf_gbdt_pack(sf_ctx* ctx, const sf_gbdt* model, void* packed);

enum { SF_SCORE_LC = 0, SF_SCORE_ENTROPY = 1 };

/* pred: [n_flows]; score: [n_flows], the chosen score rounded from binary64 to binary32;
 * margins: optional [n_flows][n_classes]; leaf_idx: optional [n_flows][n_trees] (parity checks).
 * Uses workspace for a packed copy of the trees. */
int sf_gbdt_infer(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_flows, const sf_gbdt* model,
                  int score_kind, float* margins, uint16_t* pred, float* score, uint16_t* leaf_idx);

/* The gate on such a score: flow i escalates iff score[i] > threshold.  Outputs as sf_route. */
int sf_route_score(sf_ctx* ctx, const float* score, uint32_t n_flows, float threshold, uint32_t* esc_idx,
                   uint32_t* esc_count);

/* Algorithm 1 (universal uncertainty thresholds) on a real-valued score: for each quantile q the
 * element at 1-based position ceil(q * n_flows) of the ascending order of score (device array),
 * found exactly by radix selection on the device (three histogram passes over order-preserving keys,
 * no sort, no host round trip between the passes).  host_q and host_thresholds are HOST arrays of n_q
 * entries (at most 256).  Escalating the flows with score above the
 * threshold assigns at most a fraction 1 - q of them.  Waits for the stream. */
int sf_score_quantiles(sf_ctx* ctx, const float* score, uint32_t n_flows, const double* host_q, uint32_t n_q,
                       float* host_thresholds);

/* ---- the two queues in front of the slow model ----------------------------------------------
 * Section 3.1: the flows the fast model hands on go to queue 3; the features of their later
 * packets accumulate, with their flow IDs, in queue 2; the slow model combines the two by flow
 * ID; records without a partner in the other queue are discarded after a timeout.
 *
 * Here both queues are hash tables in device memory, keyed by a 64-bit flow ID (any value but
 * 0 and 2^64-1), each record carrying a 32-bit value (for queue 3 typically the flow's row in
 * the label array, for queue 2 the row of its late-packet features) and the tick it arrived at.
 * One call is one step:
 *   1. every waiting record with now - stamp > timeout (32-bit wrap-around) is discarded;
 *   2. the arrivals of both queues are taken, stamped now; a flow ID present on both sides
 *      (waiting or just arrived) yields one pair (queue-3 value, queue-2 value) and leaves both
 *      tables; the rest waits.
 * The outcome does not depend on the order of the arrivals.  A flow ID may wait or arrive only
 * once per side; a second record of a side is dropped and counted.
 *
 * table: caller-owned device memory of sf_join_table_bytes(cap_log2) bytes, 16-byte aligned,
 * zero-filled before its first use, holding 2^cap_log2 slots per side (keep each side at most
 * half full) and, behind them, one occupancy word per 1,024 slots (a step does not sweep stretches
 * of the tables in which nothing has been stored since they were last swept).  The workspace of the context must have sf_join_workspace_bytes(cap_log2) bytes.
 * pair_q3 / pair_q2: [pair_cap], pair k = (pair_q3[k], pair_q2[k]) in no particular order;
 * *n_pairs (device) = number of pairs found (pairs beyond pair_cap are lost and counted).
 * stats: optional device array of 4 words: discarded after the timeout, arrivals that found
 * no free slot, arrivals whose flow ID was already on their side, pairs beyond pair_cap. */
typedef struct {
    void* slots;       /* device */
    uint32_t cap_log2; /* 4..28 */
} sf_join_table;

size_t sf_join_table_bytes(uint32_t cap_log2);
size_t sf_join_workspace_bytes(uint32_t cap_log2);
int sf_join_step(sf_ctx* ctx, const sf_join_table* table, uint32_t now, uint32_t timeout,
                 const uint64_t* q3_id, const uint32_t* q3_val, uint32_t n3,
                 const uint64_t* q2_id, const uint32_t* q2_val, uint32_t n2,
                 uint32_t* pair_q3, uint32_t* pair_q2, uint32_t pair_cap, uint32_t* n_pairs, uint32_t* stats);

/* The records waiting in one queue (queue = 3 or 2), in no particular order: ids, vals, stamps:
 * device arrays of cap entries (vals and stamps optional); *count (device) = number waiting. */
int sf_join_pending(sf_ctx* ctx, const sf_join_table* table, int queue, uint64_t* ids, uint32_t* vals,
                    uint32_t* stamps, uint32_t cap, uint32_t* count);

/* ---- step 5: slow model on the escalated flows only ------------------------------------
 * Sections 3.1 and 4.4: only flows the fast model is unsure of reach the slow model, and
 * its answer replaces the fast one.  The slow model is a 3-layer ReLU MLP.
 *
 * Input row of escalated flow i: feat[i][0..n_in) mapped by
 * z = clamp((x - mu) * inv_sigma, -clamp, +clamp) in binary32 (identity if mu is NULL), or,
 * when raw_src is given, the n_in = raw_pkts*raw_bits header bits of the flow read straight
 * from the packed words ({0,1}, no map).  dtype SF_BF16: z is rounded to bfloat16, the
 * weights are bfloat16, products accumulate in binary32 on the matrix cores and hidden
 * activations are rounded to bfloat16 between layers.  dtype SF_F32: all binary32.
 * label = arg-max of the logits, lowest index on ties. */
typedef struct {
    uint32_t n_in, n_h1, n_h2, n_classes;
    int dtype;                        /* SF_F32 or SF_BF16                                   */
    const float* mu;                  /* [n_in] or NULL                                      */
    const float* inv_sigma;           /* [n_in] or NULL (both or neither)                    */
    float clamp;
    const void *w1, *w2, *w3;         /* row-major [out][in]; float or bfloat16 (uint16 bit
                                         patterns) according to dtype                        */
    const float *b1, *b2, *b3;        /* [out]                                               */
    const void* ordered;              /* optional (SF_BF16 only): what sf_mlp_order wrote for these
                                         weights; NULL = re-ordered into the workspace per call */
} sf_mlp;

/* The bfloat16 kernels read the weights in MFMA operand order.  sf_mlp_order writes that copy
 * of w1, w2, w3 (sf_mlp_ordered_bytes(mlp) bytes; 0 for SF_F32) to ordered (device, 256-byte
 * aligned, caller-owned) on the context's stream; set mlp->ordered to it afterwards. */
size_t sf_mlp_ordered_bytes(const sf_mlp* mlp);
int sf_mlp_order(sf_ctx* ctx, const sf_mlp* mlp, void* ordered);

/* esc_idx / esc_count: as written by sf_route (device).  At most esc_cap flows are
 * processed (the capacity of logits; pass n_flows to process all); flows beyond it keep the
 * fast label, and the caller can see that from *esc_count > esc_cap.  logits: optional
 * [esc_cap][n_classes], row e belongs to flow esc_idx[e].  labels: [n_flows], the final
 * label of every flow: pred[i] (the fast prediction, [n_flows]) unless flow i escalated,
 * then the slow label.  pred may be NULL (or equal to labels) when the caller has already
 * filled labels with the fast prediction.  Exactly one of feat / raw_src is given.
 * Uses workspace for hidden activations. */
int sf_slow_infer(sf_ctx* ctx, const float* feat, uint32_t feat_ld, const sf_packets* raw_src,
                  const sf_feat_cfg* raw_cfg, const uint32_t* esc_idx,
                  const uint32_t* esc_count, uint32_t esc_cap, uint32_t n_flows,
                  const sf_mlp* mlp, const uint16_t* pred, float* logits, uint16_t* labels);

/* The slow model behind the queue join (Section 3.1: it combines the features of the later
 * packets with the flow handed on by the fast model): pair k reads row pair_row[k] of feat
 * ([n_rows][feat_ld], e.g. the late-packet features; entries >= n_rows are clamped) and writes
 * its label to labels[pair_flow[k]] ([n_flows]; entries >= n_flows are skipped).  pair_row,
 * pair_flow, n_pairs: device, as written by sf_join_step (its pair_q2, pair_q3, n_pairs); at
 * most pair_cap pairs are processed.  logits: optional [pair_cap][n_classes], row k = pair k. */
int sf_slow_infer_pairs(sf_ctx* ctx, const float* feat, uint32_t feat_ld, uint32_t n_rows,
                        const uint32_t* pair_row, const uint32_t* pair_flow, const uint32_t* n_pairs,
                        uint32_t pair_cap, uint32_t n_flows, const sf_mlp* mlp, float* logits, uint16_t* labels);

/* ---- steps 1-3 in one kernel, all four steps in one call ----------------------------------------
 * Sections 3.1 and 3.2: features from the first k packets, the fast model on every flow, the gate, the slow
 * model on the flows the gate hands on.
 *
 * sf_featurize_fast_infer: the results of sf_featurize followed by sf_fast_infer (pred, top_votes), but for
 * window depths up to 16 packets and forests that run one lane per flow both steps are ONE kernel that
 * builds each tile of flows' features in shared memory and walks the forest there.  The feature matrix is
 * then written only where the slow model will read it: row i of feat is written iff flow i escalates under
 * the gate given by host_vmin / n_vmin (as sf_route: top_votes < vmin, or vmin[pred]); the other rows are
 * left untouched.  feat = NULL: no row is written (a slow model that reads header bits needs none).
 * Other shapes run the separate kernels and write every row (they need feat).  labels: optional
 * [n_flows]; labels[i] = pred[i], the start of the final label array (pass it to sf_slow_infer with
 * pred = NULL).
 *
 * sf_classify: all four steps: sf_featurize_fast_infer, sf_route, sf_slow_infer (with pred given and
 * esc_cap = n_flows); the results are those of the four calls in turn with the same arguments, except for
 * the rows of feat that are not written.  cfg->raw_pkts > 0: the slow model reads the header bits of pk
 * (raw_pkts * raw_bits = mlp->n_in) and no feature row is kept.  logits: optional [n_flows][n_classes],
 * row e belongs to flow esc_idx[e].  Both use workspace as the separate calls do. */
int sf_featurize_fast_infer(sf_ctx* ctx, const sf_packets* pk, const sf_feat_cfg* cfg, const sf_forest* forest,
                            const uint16_t* host_vmin, uint32_t n_vmin, float* feat, uint32_t feat_ld,
                            uint16_t* pred, uint16_t* top_votes, uint16_t* labels);
int sf_classify(sf_ctx* ctx, const sf_packets* pk, const sf_feat_cfg* cfg, const sf_forest* forest,
                const uint16_t* host_vmin, uint32_t n_vmin, const sf_mlp* mlp, float* feat, uint32_t feat_ld,
                uint16_t* pred, uint16_t* top_votes, uint32_t* esc_idx, uint32_t* esc_count, float* logits,
                uint16_t* labels);

/* ---- measurement aid ---------------------------------------------------------------------------
 * Not a step of the method.  The walk of the fast model (Section 3.1: it sees every flow, so it sets the
 * service rate) is bound by gathers, not by memory bandwidth; sf_probe_gather measures what such gathers
 * cost on the device at hand, so that a benchmark can price the walk against them.  One launch of `blocks`
 * blocks of 256 lanes; every lane runs eight chains of `iters` dependent gathers.  kind 0: shared memory,
 * 4 bytes, the lane's own column at a data-dependent row; kind 1: shared memory, 16 bytes at a
 * data-dependent record; kind 2: global memory through the caches, 16 bytes at a data-dependent record of
 * `table`.  table: device, 16-byte aligned, 16 << table_log2 bytes (12 <= table_log2 <= 24; kind 2: from 8) of arbitrary
 * words, read only; sink: device, [blocks * 256] words, written.  *host_wave_gathers (optional) = number
 * of 64-lane gathers the launch performs; time it with events on the context's stream. */
int sf_probe_gather(sf_ctx* ctx, int kind, uint32_t table_log2, uint32_t iters, uint32_t blocks,
                    const void* table, uint32_t* sink, uint64_t* host_wave_gathers);

#ifdef __cplusplus
}
#endif
#endif /* SERVEFLOW_H */
