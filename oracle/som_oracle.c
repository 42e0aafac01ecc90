/*
 * CPU oracle for one batch-mode self-organizing-map training epoch.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the paper's method computes.  It is used by the tests, by the smoke
 * check and by the benchmark's reported CPU baseline; the product path (the
 * HIP library) never calls it and shares no code, header, table or constant
 * with it.
 *
 * What is followed (paper: "Self-organizing maps in batch mode"):
 *   - best matching unit: the node whose weight vector is nearest to the
 *     instance (the BMU equation and the inequality that follows it), with the
 *     Euclidean distance the GPU section opts for; ties go to the lowest node
 *     index;
 *   - Gaussian neighbourhood of the grid distance between two nodes (the
 *     neighbourhood equation), read as exp(-d^2 / (2 r^2)) with r the cooled
 *     radius;
 *   - batch update (the batch equation): each new weight vector is the
 *     neighbourhood-weighted mean of all instances;
 *   - U-matrix (the U-matrix equation): mean Euclidean distance between a node's
 *     weight vector and those of its immediate grid neighbours;
 *   - radius / learning-rate cooling, linear or exponential (options -t/-T,
 *     -r/-R, -l/-L of the command-line interface);
 *   - map type planar or toroid (-m), grid type square or hexagonal (-g).
 *
 * Every sum is taken in double precision in the order the definition states.
 * No blocking, no separable filters, no expansion of the squared distance.
 * Node index i = y * cols + x (x = column, y = row); the code book is
 * node-major [rows*cols][dim], single precision, as in the paper's API.
 *
 * Parity pins (tests marked "not gpu"): brute force in numpy on tiny inputs,
 * k-means limit for radius -> 0, global-mean limit for radius -> infinity,
 * torus translation symmetry, zero-mass nodes keep their weights, closed-form
 * U-matrix of a ramp, sparse == densified dense, cooling end points; distances to
 * the BMU: right triangles, agreement with the minimum the BMU search reports,
 * scaling, numpy on tiny inputs.
 * Parity against the original tool's outputs: parity unpinned (no source, no
 * data and no printed numerical example are available).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_PLANAR = 0, ORACLE_TOROID = 1 };
enum { ORACLE_SQUARE = 0, ORACLE_HEXAGONAL = 1 };
enum { ORACLE_LINEAR = 0, ORACLE_EXPONENTIAL = 1 };
enum { ORACLE_GAUSSIAN = 0, ORACLE_BUBBLE = 1 };

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------------------
 * Grid geometry (paper: each neuron has two coordinates in a grid; options -g
 * and -m).  Square grid: node (x, y) sits at (x, y).  Hexagonal grid: odd rows
 * are shifted right by half a cell and rows are sqrt(3)/2 apart, so that all
 * six neighbours of an interior node are at distance exactly 1.
 *
 * Returned value: q = 4 * (squared grid distance), an exact integer:
 *   a = |yi - yb|,  m = |2 (xi - xb) + hex * ((yi mod 2) - (yb mod 2))|
 *   toroid: a = min(a, rows - a), m = min(m, 2 cols - m)
 *   q = m^2 + 4 a^2 (square)   or   m^2 + 3 a^2 (hexagonal)
 * ------------------------------------------------------------------------- */
int64_t oracle_grid_q(int rows, int cols, int map_type, int grid_type, int i, int b)
{
    int xi = i % cols, yi = i / cols;
    int xb = b % cols, yb = b / cols;
    int64_t a = llabs((long long)yi - yb);
    int64_t m = 2 * ((int64_t)xi - xb);
    if (grid_type == ORACLE_HEXAGONAL)
        m += (yi % 2) - (yb % 2);
    m = llabs(m);
    if (map_type == ORACLE_TOROID) {
        if (rows - a < a) a = rows - a;
        if (2 * (int64_t)cols - m < m) m = 2 * (int64_t)cols - m;
    }
    return m * m + (grid_type == ORACLE_HEXAGONAL ? 3 : 4) * a * a;
}

/* Gaussian neighbourhood: exp(-d^2 / (2 r^2)) = exp(-q / (8 r^2)). */
double oracle_neighbourhood(int rows, int cols, int map_type, int grid_type,
                            int i, int b, double radius)
{
    double q = (double)oracle_grid_q(rows, cols, map_type, grid_type, i, b);
    return exp(-q / (8.0 * radius * radius));
}

/*
 * The other neighbourhoods of the command line (options -n and -p): function 0 = Gaussian,
 * 1 = bubble (weight 1 inside the current radius, 0 outside); compact != 0 cuts the Gaussian
 * off beyond the current radius (the bubble has compact support by definition).  "Inside the
 * radius" means grid distance d <= r, that is q = 4 d^2 <= 4 r^2, compared in double.
 */
double oracle_neighbourhood_kind(int rows, int cols, int map_type, int grid_type,
                                 int i, int b, double radius, int function, int compact)
{
    double q = (double)oracle_grid_q(rows, cols, map_type, grid_type, i, b);
    int inside = q <= 4.0 * radius * radius;
    if (function == ORACLE_BUBBLE) return inside ? 1.0 : 0.0;
    if (compact && !inside) return 0.0;
    return exp(-q / (8.0 * radius * radius));
}

/* ---------------------------------------------------------------------------
 * Squared Euclidean distance between a dense instance and a weight vector.
 * ------------------------------------------------------------------------- */
static double sqdist_dense(const float *x, const float *w, int dim)
{
    double s = 0.0;
    for (int c = 0; c < dim; ++c) {
        double d = (double)x[c] - (double)w[c];
        s += d * d;
    }
    return s;
}

/* Same distance for a sparse instance, by the same definition: the sum runs over
 * all dim coordinates in ascending order, a coordinate the row does not list
 * counts as zero.  idx holds the row's columns, zero-based and strictly
 * increasing (the sparse file format of the command-line interface), so one
 * cursor into the row tells for every coordinate whether it is listed.  No
 * regrouping: the result has the bits sqdist_dense gives on the densified row,
 * and it is exactly 0 when the instance coincides with the weight vector. */
static double sqdist_csr(const int32_t *idx, const float *val, int64_t len,
                         const float *w, int dim)
{
    double s = 0.0;
    int64_t p = 0;
    for (int c = 0; c < dim; ++c) {
        double x = 0.0;
        if (p < len && idx[p] == c) { x = (double)val[p]; ++p; }
        double d = x - (double)w[c];
        s += d * d;
    }
    return s;
}

/* ---------------------------------------------------------------------------
 * Best matching units (BMU equation): bmu[j] = the smallest node index whose
 * squared distance to instance j equals the minimum over all nodes.
 * d2min (may be NULL) receives that minimum.
 * ------------------------------------------------------------------------- */
void oracle_bmu_dense(const float *X, int64_t n, int dim, const float *W, int k,
                      int32_t *bmu, double *d2min)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        const float *x = X + j * (int64_t)dim;
        double best = INFINITY;
        int32_t arg = 0;
        for (int i = 0; i < k; ++i) {
            double d2 = sqdist_dense(x, W + (int64_t)i * dim, dim);
            if (d2 < best) { best = d2; arg = i; }
        }
        bmu[j] = arg;
        if (d2min) d2min[j] = best;
    }
}

void oracle_bmu_csr(const int64_t *indptr, const int32_t *indices, const float *values,
                    int64_t n, int dim, const float *W, int k, int32_t *bmu, double *d2min)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t j = 0; j < n; ++j) {
        int64_t s = indptr[j], len = indptr[j + 1] - indptr[j];
        double best = INFINITY;
        int32_t arg = 0;
        for (int i = 0; i < k; ++i) {
            double d2 = sqdist_csr(indices + s, values + s, len, W + (int64_t)i * dim, dim);
            if (d2 < best) { best = d2; arg = i; }
        }
        bmu[j] = arg;
        if (d2min) d2min[j] = best;
    }
}

/* Squared distances of chosen (instance, node) pairs: what a parity test needs
 * to place another implementation's answer inside or outside the near-tie band. */
void oracle_sqdist_pairs_dense(const float *X, int dim, const float *W, int64_t npairs,
                               const int64_t *inst, const int32_t *node, double *out)
{
    for (int64_t p = 0; p < npairs; ++p)
        out[p] = sqdist_dense(X + inst[p] * (int64_t)dim, W + (int64_t)node[p] * dim, dim);
}

void oracle_sqdist_pairs_csr(const int64_t *indptr, const int32_t *indices, const float *values,
                             int dim, const float *W, int64_t npairs,
                             const int64_t *inst, const int32_t *node, double *out)
{
    for (int64_t p = 0; p < npairs; ++p) {
        int64_t s = indptr[inst[p]], len = indptr[inst[p] + 1] - s;
        out[p] = sqdist_csr(indices + s, values + s, len, W + (int64_t)node[p] * dim, dim);
    }
}

/* ---------------------------------------------------------------------------
 * Post-training outputs.  The paper lists the BMU of every instance, the code
 * book and the U-matrix as results (output prefix of the command line, class
 * variables of the Python interface) and prints no formula for a quality
 * figure.  Reading taken here: dist[j] = Euclidean distance between instance j
 * and the weight vector of node bmu[j]; the return value is their mean, the
 * quantisation error in its usual sense (0 for n = 0).  dist may be NULL.
 * ------------------------------------------------------------------------- */
double oracle_bmu_distances_dense(const float *X, int64_t n, int dim, const float *W,
                                  const int32_t *bmu, double *dist)
{
    double total = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        double d = sqrt(sqdist_dense(X + j * (int64_t)dim, W + (int64_t)bmu[j] * dim, dim));
        if (dist) dist[j] = d;
        total += d;
    }
    return n > 0 ? total / (double)n : 0.0;
}

double oracle_bmu_distances_csr(const int64_t *indptr, const int32_t *indices, const float *values,
                                int64_t n, int dim, const float *W, const int32_t *bmu, double *dist)
{
    double total = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        int64_t s = indptr[j], len = indptr[j + 1] - s;
        double d = sqrt(sqdist_csr(indices + s, values + s, len, W + (int64_t)bmu[j] * dim, dim));
        if (dist) dist[j] = d;
        total += d;
    }
    return n > 0 ? total / (double)n : 0.0;
}

/* ---------------------------------------------------------------------------
 * Batch update (batch equation).  The neighbourhood weight of instance j for
 * node i depends on j only through bmu[j], so the sums over instances regroup
 * exactly into sums over BMU nodes:
 *     S[b] = sum of the instances whose BMU is b,  C[b] = their number,
 *     N[i] = sum_b h(b, i) S[b],   D[i] = sum_b h(b, i) C[b],   w_i = N[i] / D[i].
 * ------------------------------------------------------------------------- */
void oracle_accumulate_dense(const float *X, int64_t n, int dim, const int32_t *bmu, int k,
                             double *S, double *C)
{
    memset(S, 0, sizeof(double) * (size_t)k * dim);
    memset(C, 0, sizeof(double) * (size_t)k);
    for (int64_t j = 0; j < n; ++j) {
        double *s = S + (int64_t)bmu[j] * dim;
        const float *x = X + j * (int64_t)dim;
        for (int c = 0; c < dim; ++c) s[c] += (double)x[c];
        C[bmu[j]] += 1.0;
    }
}

void oracle_accumulate_csr(const int64_t *indptr, const int32_t *indices, const float *values,
                           int64_t n, int dim, const int32_t *bmu, int k, double *S, double *C)
{
    memset(S, 0, sizeof(double) * (size_t)k * dim);
    memset(C, 0, sizeof(double) * (size_t)k);
    for (int64_t j = 0; j < n; ++j) {
        double *s = S + (int64_t)bmu[j] * dim;
        for (int64_t p = indptr[j]; p < indptr[j + 1]; ++p) s[indices[p]] += (double)values[p];
        C[bmu[j]] += 1.0;
    }
}

/*
 * New weight vector of one node from the per-node sums.  `scale` (the learning rate the API
 * carries) multiplies the neighbourhood weight in numerator and denominator alike, exactly
 * as a constant factor on h would in the batch equation, and so cancels.  A node whose
 * unscaled neighbourhood mass D is below eps_mass keeps its weights (no instance
 * influences it).  `w` is node i's own weight vector (in/out).  Returns D.  `num` is scratch
 * of dim doubles.
 */
static double update_node(int i, const double *S, const double *C, float *w, int rows, int cols,
                          int dim, int map_type, int grid_type, double radius, double scale,
                          double eps_mass, double *num, int function, int compact)
{
    int k = rows * cols;
    double den = 0.0, mass = 0.0;
    for (int c = 0; c < dim; ++c) num[c] = 0.0;
    for (int b = 0; b < k; ++b) {
        if (C[b] == 0.0) continue;          /* contributes exact zeros */
        double h = oracle_neighbourhood_kind(rows, cols, map_type, grid_type, i, b, radius, function,
                                             compact);
        const double *s = S + (int64_t)b * dim;
        mass += h * C[b];
        den += scale * h * C[b];
        for (int c = 0; c < dim; ++c) num[c] += scale * h * s[c];
    }
    if (mass >= eps_mass)
        for (int c = 0; c < dim; ++c) w[c] = (float)(num[c] / den);
    return mass;
}

/*
 * New code book for all nodes.  D_out (may be NULL) receives the masses.  W is read and
 * written in place: node i's new vector depends on S and C only.
 */
void oracle_update_kind(const double *S, const double *C, float *W, int rows, int cols, int dim,
                        int map_type, int grid_type, double radius, double scale,
                        double eps_mass, double *D_out, int function, int compact)
{
    int k = rows * cols;
#pragma omp parallel
    {
        double *num = (double *)malloc(sizeof(double) * (size_t)dim);
#pragma omp for schedule(dynamic, 4)
        for (int i = 0; i < k; ++i) {
            double mass = update_node(i, S, C, W + (int64_t)i * dim, rows, cols, dim, map_type,
                                      grid_type, radius, scale, eps_mass, num, function, compact);
            if (D_out) D_out[i] = mass;
        }
        free(num);
    }
}

void oracle_update(const double *S, const double *C, float *W, int rows, int cols, int dim,
                   int map_type, int grid_type, double radius, double scale,
                   double eps_mass, double *D_out)
{
    oracle_update_kind(S, C, W, rows, cols, dim, map_type, grid_type, radius, scale, eps_mass, D_out,
                       ORACLE_GAUSSIAN, 0);
}

/*
 * The same for a chosen subset of nodes (sampled checks on maps too large to update whole):
 * W_out[t] receives the new vector of node nodes[t] (or its old vector from W if its mass is
 * below eps_mass), D_out[t] its mass.  W itself is not modified.
 */
void oracle_update_nodes(const double *S, const double *C, const float *W, int rows, int cols,
                         int dim, int map_type, int grid_type, double radius, double scale,
                         double eps_mass, const int32_t *nodes, int n_nodes, float *W_out,
                         double *D_out)
{
#pragma omp parallel
    {
        double *num = (double *)malloc(sizeof(double) * (size_t)dim);
        float *row = (float *)malloc(sizeof(float) * (size_t)dim);
#pragma omp for schedule(dynamic, 1)
        for (int t = 0; t < n_nodes; ++t) {
            int i = nodes[t];
            memcpy(row, W + (int64_t)i * dim, sizeof(float) * (size_t)dim);
            double mass = update_node(i, S, C, row, rows, cols, dim, map_type, grid_type, radius,
                                      scale, eps_mass, num, ORACLE_GAUSSIAN, 0);
            memcpy(W_out + (int64_t)t * dim, row, sizeof(float) * (size_t)dim);
            if (D_out) D_out[t] = mass;
        }
        free(num);
        free(row);
    }
}

/* One whole epoch on dense data: BMUs against the incoming code book, then the
 * batch update in place.  Returns 0, or 1 if memory could not be obtained. */
int oracle_epoch_dense(const float *X, int64_t n, int dim, float *W, int rows, int cols,
                       int map_type, int grid_type, double radius, double scale,
                       double eps_mass, int32_t *bmu)
{
    int k = rows * cols;
    double *S = (double *)malloc(sizeof(double) * (size_t)k * dim);
    double *C = (double *)malloc(sizeof(double) * (size_t)k);
    if (!S || !C) { free(S); free(C); return 1; }
    oracle_bmu_dense(X, n, dim, W, k, bmu, NULL);
    oracle_accumulate_dense(X, n, dim, bmu, k, S, C);
    oracle_update(S, C, W, rows, cols, dim, map_type, grid_type, radius, scale, eps_mass, NULL);
    free(S); free(C);
    return 0;
}

int oracle_epoch_csr(const int64_t *indptr, const int32_t *indices, const float *values,
                     int64_t n, int dim, float *W, int rows, int cols, int map_type,
                     int grid_type, double radius, double scale, double eps_mass, int32_t *bmu)
{
    int k = rows * cols;
    double *S = (double *)malloc(sizeof(double) * (size_t)k * dim);
    double *C = (double *)malloc(sizeof(double) * (size_t)k);
    if (!S || !C) { free(S); free(C); return 1; }
    oracle_bmu_csr(indptr, indices, values, n, dim, W, k, bmu, NULL);
    oracle_accumulate_csr(indptr, indices, values, n, dim, bmu, k, S, C);
    oracle_update(S, C, W, rows, cols, dim, map_type, grid_type, radius, scale, eps_mass, NULL);
    free(S); free(C);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Cooling (options -t/-T with -r/-R and -l/-L): the value used in epoch e of E,
 * e = 0 .. E-1, moving from v0 (first epoch) to vN (last epoch).
 *   linear:      v0 + (vN - v0) e / (E - 1)
 *   exponential: v0 (vN / v0)^(e / (E - 1))
 * A single epoch uses v0.
 * ------------------------------------------------------------------------- */
double oracle_cool(double v0, double vN, int n_epochs, int epoch, int kind)
{
    if (n_epochs <= 1) return v0;
    double t = (double)epoch / (double)(n_epochs - 1);
    if (kind == ORACLE_EXPONENTIAL) return v0 * pow(vN / v0, t);
    return v0 + (vN - v0) * t;
}

/* ---------------------------------------------------------------------------
 * U-matrix (U-matrix equation): for every node, the mean Euclidean distance
 * between its weight vector and those of its immediate neighbours, i.e. the
 * other nodes at grid distance <= 1 (q <= 4): up to four on a square grid, up
 * to six on a hexagonal one, fewer on the border of a planar map.  A node with
 * no neighbour (1x1 map) gets 0.
 * ------------------------------------------------------------------------- */
void oracle_umatrix(const float *W, int rows, int cols, int dim, int map_type, int grid_type,
                    double *U)
{
    int k = rows * cols;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < k; ++j) {
        double sum = 0.0;
        int cnt = 0;
        for (int i = 0; i < k; ++i) {
            if (i == j) continue;
            if (oracle_grid_q(rows, cols, map_type, grid_type, i, j) > 4) continue;
            sum += sqrt(sqdist_dense(W + (int64_t)i * dim, W + (int64_t)j * dim, dim));
            ++cnt;
        }
        U[j] = cnt ? sum / cnt : 0.0;
    }
}
