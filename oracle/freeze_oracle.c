/*
 * CPU oracle for the Freeze Inference per-layer cache lookup.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition the HIP library
 * is checked against; it is compiled on its own, shares no code, header or
 * table with the library, and is reached only from the tests, the smoke check
 * and the benchmark's cpu_baseline leg.  Nothing here is tuned.
 *
 * What it computes (paper Sec. 3, the cache look-up API; Sec. 2.1, approximate
 * caching): for a query vector, the k cached entries of a layer nearest in
 * Euclidean distance, each with its label and distance; from these the label
 * held by most of the k neighbours (m_i occurrences, share S_i = m_i / k) and
 * whether the look-up is a hit, i.e. whether the agreement reaches the layer's
 * threshold.  Pseudocode 1 (FreezeInference) gives the cascade: layers are
 * tried in order and the first hit ends the request.  Sec. 5 ("Freeze
 * Inference on GPUs") asks for the batch to be rebuilt without the frozen
 * items after each layer: fz_oracle_compact is that step.
 *
 * Readings taken where the paper is silent:
 *   - distance: Euclidean; the squared distance is what is reported and ranked
 *     (same ranking), D[n] = sum_i (q_i - c_{n,i})^2 in double, i ascending;
 *   - equal distances: the lower entry index ranks first;
 *   - label decision: plain count, equal counts -> the smaller label id;
 *   - hit: votes >= vote_threshold (integer agreement threshold);
 *   - the cache values are the values as stored (bf16 bit patterns widen
 *     exactly); queries are fp32 and are never rounded;
 *   - no layer hits -> label -1, exit layer -1 (the model's own output layer
 *     would decide; the model is outside this path).
 * The distance-weighted confidence of Sec. 3 (C_i = S_i * sum_j 1/d_j) is
 * computed by fz_oracle_confidence; the look-up, cascade and ComputeThresholds
 * (Pseudocode 1) built on it are in freeze_oracle.py.  Readings for that rule:
 * d_j is the Euclidean distance (square root of the squared distance); a zero
 * distance gives +inf, i.e. always a hit; equal confidences -> the smaller
 * label id; hit iff confidence > threshold (strict, as the pseudocode writes
 * it), the confidence rounded once to fp32 and compared in fp32; the running
 * maximum of ComputeThresholds starts at 0.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <unistd.h>

enum { FZO_F32 = 0, FZO_BF16 = 1 };

static double widen(const void *entries, int kind, int64_t pos)
{
    if (kind == FZO_F32)
        return (double)((const float *)entries)[pos];
    /* bf16 is the upper half of an IEEE binary32 */
    uint32_t bits = (uint32_t)((const uint16_t *)entries)[pos] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Squared Euclidean distance between one query and one cached entry. */
static double sqdist(const float *q, const void *entries, int kind, int64_t row, int64_t d)
{
    double acc = 0.0;
    for (int64_t i = 0; i < d; ++i) {
        double diff = (double)q[i] - widen(entries, kind, row * d + i);
        acc += diff * diff;
    }
    return acc;
}

/* k nearest entries of one query under the order (D, index); out arrays have k slots. */
static void knn_one(const float *q, const void *entries, int kind, int64_t n, int64_t d, int k,
                    int32_t *out_idx, double *out_dist)
{
    int have = 0;
    for (int64_t row = 0; row < n; ++row) {
        double D = sqdist(q, entries, kind, row, d);
        if (have == k && !(D < out_dist[k - 1]))
            continue; /* not better than the current k-th; on equality the earlier index stays */
        int pos = (have < k) ? have : k - 1;
        /* move past every kept entry with a larger distance (equal ones keep their place) */
        while (pos > 0 && out_dist[pos - 1] > D) {
            out_dist[pos] = out_dist[pos - 1];
            out_idx[pos] = out_idx[pos - 1];
            --pos;
        }
        out_dist[pos] = D;
        out_idx[pos] = (int32_t)row;
        if (have < k)
            ++have;
    }
}

/* Label vote over k neighbour labels: most frequent label, smaller id on equal counts. */
static void vote_one(const int32_t *labels, const int32_t *nbr, int k, int num_classes,
                     int vote_threshold, int32_t *label, int32_t *votes, uint8_t *hit)
{
    int32_t best_label = -1, best_count = 0;
    for (int32_t c = 0; c < num_classes; ++c) {
        int32_t m = 0;
        for (int j = 0; j < k; ++j)
            if (labels[nbr[j]] == c)
                ++m;
        if (m > best_count) { /* strict: the first (smallest) label wins a tie */
            best_count = m;
            best_label = c;
        }
    }
    *label = best_label;
    *votes = best_count;
    *hit = (uint8_t)(best_count >= vote_threshold);
}

struct knn_job {
    const float *q;
    const void *entries;
    int kind;
    int64_t b, n, d;
    int k;
    int32_t *idx;
    double *dist;
    int tid, nthreads;
};

static void *knn_worker(void *p)
{
    struct knn_job *j = (struct knn_job *)p;
    for (int64_t i = j->tid; i < j->b; i += j->nthreads)
        knn_one(j->q + i * j->d, j->entries, j->kind, j->n, j->d, j->k,
                j->idx + i * j->k, j->dist + i * j->k);
    return NULL;
}

int fz_oracle_host_threads(void)
{
    long c = sysconf(_SC_NPROCESSORS_ONLN);
    return c < 1 ? 1 : (int)c;
}

/*
 * Exact k-NN of b queries against n entries (Sec. 3: "computes k-nearest
 * neighbors on the input and obtains a set of k tuples").
 * queries [b,d] fp32; entries [n,d] fp32 or bf16 bits; out_idx [b,k]; out_dist
 * [b,k] squared distances in double, ascending in (dist, idx).
 * nthreads <= 0 -> all online cores.  Returns the number of threads used, or -1.
 */
int fz_oracle_knn(const float *queries, int64_t b, const void *entries, int kind, int64_t n,
                  int64_t d, int k, int32_t *out_idx, double *out_dist, int nthreads)
{
    if (!queries || !entries || !out_idx || !out_dist || b < 0 || n < 1 || d < 1 || k < 1 || k > n ||
        (kind != FZO_F32 && kind != FZO_BF16))
        return -1;
    if (nthreads <= 0)
        nthreads = fz_oracle_host_threads();
    if (nthreads > b)
        nthreads = b > 0 ? (int)b : 1;
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
    struct knn_job *jobs = (struct knn_job *)malloc(sizeof(struct knn_job) * (size_t)nthreads);
    for (int t = 0; t < nthreads; ++t) {
        struct knn_job j = {queries, entries, kind, b, n, d, k, out_idx, out_dist, t, nthreads};
        jobs[t] = j;
        pthread_create(&th[t], NULL, knn_worker, &jobs[t]);
    }
    for (int t = 0; t < nthreads; ++t)
        pthread_join(th[t], NULL);
    free(th);
    free(jobs);
    return nthreads;
}

/*
 * Vote and hit decision for b neighbour lists (Sec. 3: m_i occurrences of label
 * n_i among the k neighbours; Sec. 2.1: hit if the agreement reaches the threshold).
 */
int fz_oracle_vote(const int32_t *labels, const int32_t *nbr_idx, int64_t b, int k, int num_classes,
                   int vote_threshold, int32_t *out_label, int32_t *out_votes, uint8_t *out_hit)
{
    if (!labels || !nbr_idx || !out_label || !out_votes || !out_hit || k < 1 || num_classes < 1)
        return -1;
    for (int64_t i = 0; i < b; ++i)
        vote_one(labels, nbr_idx + i * k, k, num_classes, vote_threshold, out_label + i,
                 out_votes + i, out_hit + i);
    return 0;
}

/*
 * The paper's distance-weighted confidence (Sec. 3): for each label i with m_i
 * neighbours at distances d_1..d_{m_i}, C_i = (m_i / k) * sum_j 1/d_j with
 * d = sqrt(squared distance); the predicted label maximises C_i (smaller id on
 * equality); a zero distance gives +inf.  nbr_dist holds squared distances.
 */
int fz_oracle_confidence(const int32_t *labels, const int32_t *nbr_idx, const double *nbr_dist,
                         int64_t b, int k, int num_classes, int32_t *out_label, double *out_conf)
{
    if (!labels || !nbr_idx || !nbr_dist || !out_label || !out_conf || k < 1 || num_classes < 1)
        return -1;
    for (int64_t i = 0; i < b; ++i) {
        int32_t best = -1;
        double best_c = -1.0;
        for (int32_t c = 0; c < num_classes; ++c) {
            int m = 0;
            double inv = 0.0;
            for (int j = 0; j < k; ++j)
                if (labels[nbr_idx[i * k + j]] == c) {
                    ++m;
                    inv += 1.0 / sqrt(nbr_dist[i * k + j]);
                }
            if (m == 0)
                continue;
            double C = ((double)m / (double)k) * inv;
            if (C > best_c) {
                best_c = C;
                best = c;
            }
        }
        out_label[i] = best;
        out_conf[i] = best_c;
    }
    return 0;
}

/*
 * Batch reconstruction (Sec. 5): the ids in sel_in[0..count) whose hit flag is
 * 0, in their original order.  hit[j] belongs to sel_in[j].  Returns the count.
 */
int64_t fz_oracle_compact(const uint8_t *hit, const int32_t *sel_in, int64_t count, int32_t *sel_out)
{
    int64_t m = 0;
    for (int64_t j = 0; j < count; ++j)
        if (!hit[j])
            sel_out[m++] = sel_in[j];
    return m;
}

struct cascade_job {
    int num_layers;
    const float *const *queries;
    const void *const *entries;
    const int *kinds;
    const int64_t *ns, *ds;
    const int32_t *const *labels;
    const int *num_classes;
    int k;
    const int *thresholds;
    int64_t b;
    int32_t *out_label, *out_exit;
    int tid, nthreads;
};

static void *cascade_worker(void *p)
{
    struct cascade_job *j = (struct cascade_job *)p;
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)j->k);
    double *dist = (double *)malloc(sizeof(double) * (size_t)j->k);
    for (int64_t i = j->tid; i < j->b; i += j->nthreads) {
        j->out_label[i] = -1;
        j->out_exit[i] = -1;
        for (int l = 0; l < j->num_layers; ++l) { /* Pseudocode 1: layers in order */
            knn_one(j->queries[l] + i * j->ds[l], j->entries[l], j->kinds[l], j->ns[l], j->ds[l], j->k,
                    idx, dist);
            int32_t label, votes;
            uint8_t hit;
            vote_one(j->labels[l], idx, j->k, j->num_classes[l], j->thresholds[l], &label, &votes, &hit);
            if (hit) { /* freeze: return the cached prediction, skip the remaining layers */
                j->out_label[i] = label;
                j->out_exit[i] = l;
                break;
            }
        }
    }
    free(idx);
    free(dist);
    return NULL;
}

/*
 * FreezeInference of Pseudocode 1 restricted to the look-ups: request i carries
 * one query per layer (row i of queries[l]); the first layer whose look-up hits
 * gives (label, exit layer); hits_per_layer[l] counts the requests frozen at l.
 */
int fz_oracle_cascade(int num_layers, const float *const *queries, int64_t b,
                      const void *const *entries, const int *kinds, const int64_t *ns,
                      const int64_t *ds, const int32_t *const *labels, const int *num_classes, int k,
                      const int *thresholds, int32_t *out_label, int32_t *out_exit,
                      int64_t *hits_per_layer, int nthreads)
{
    if (num_layers < 1 || b < 0 || k < 1)
        return -1;
    for (int l = 0; l < num_layers; ++l)
        if (k > ns[l])
            return -1;
    if (nthreads <= 0)
        nthreads = fz_oracle_host_threads();
    if (nthreads > b)
        nthreads = b > 0 ? (int)b : 1;
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
    struct cascade_job *jobs = (struct cascade_job *)malloc(sizeof(struct cascade_job) * (size_t)nthreads);
    for (int t = 0; t < nthreads; ++t) {
        struct cascade_job j = {num_layers, queries, entries, kinds, ns, ds, labels, num_classes,
                                k, thresholds, b, out_label, out_exit, t, nthreads};
        jobs[t] = j;
        pthread_create(&th[t], NULL, cascade_worker, &jobs[t]);
    }
    for (int t = 0; t < nthreads; ++t)
        pthread_join(th[t], NULL);
    free(th);
    free(jobs);
    for (int l = 0; l < num_layers; ++l)
        hits_per_layer[l] = 0;
    for (int64_t i = 0; i < b; ++i)
        if (out_exit[i] >= 0)
            ++hits_per_layer[out_exit[i]];
    return nthreads;
}
