/*
 * CPU ORACLE FOR CTC -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, slow, double-precision implementation of the Connectionist Temporal
 * Classification cost and of its gradient with respect to the pre-softmax
 * activations.  It exists so that the GPU library can be checked against
 * something independent: it shares no code, header, table or helper with the
 * HIP path, and only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.
 *
 * What it computes (Section 3.3, Eq. (ctc); output softmax of Section 3.1;
 * the two-pass structure of Appendix "GPU Implementation of CTC Loss Function"):
 * for each utterance b on its own, with y_t(k) the softmax over k of x[t,b,:],
 *
 *     p_b   = sum over all alignments pi of label_b to T_b frames of prod_t y_t(pi_t)
 *     cost  = -ln p_b
 *     grad[t,b,k] = d cost / d x[t,b,k] = y_t(k) - (1/p_b) * (mass of alignments with pi_t = k)
 *
 * An alignment is a length-T_b string over the alphabet that gives the label
 * after merging runs of equal symbols and then deleting blanks (the CTC
 * operator of Graves et al. that the paper's Align(x, y) refers to).
 *
 * The sum is evaluated with the forward/backward dynamic programme over the
 * blank-interleaved label (S = 2L+1 lattice states), entirely in natural-log
 * space, with an addition that skips -inf operands as the appendix describes.
 * No blocking, fusion or reordering: softmax, alpha, beta, gradient, one
 * utterance after the other (utterances are spread over OpenMP threads, one
 * utterance per thread at a time, which is the paper's CPU design).
 *
 * Conventions where the paper is silent:
 *   - beta is "exclusive": it does not contain the emission at its own frame, so
 *     ln alpha_t(s) + ln beta_t(s) is the log mass of alignments through (t, s).
 *   - an utterance with no valid alignment (too few frames) has cost +inf and an
 *     all-zero gradient; frames t >= T_b are never read and get zero gradient.
 *   - T_b = 0: the empty product, cost 0 for an empty label and +inf otherwise.
 *
 * Pins (tests/test_oracle_pins.py): brute-force enumeration of every alignment,
 * sum over all labelings = 1, finite differences, closed forms, alignment
 * counts under uniform logits, reversal and relabelling symmetries, and a
 * library CTC routine.
 *
 * Second function, ctc_oracle_best_path: the single most probable alignment
 *     l* = argmax over alignments pi of prod_t y_t(pi_t)
 * (Section 5.1, "Dataset Construction": the alignment step of the segmentation
 * pipeline, which the paper calls essentially a Viterbi alignment), by the
 * same lattice with max in place of the sum and a table of predecessors.
 * Pins (tests/test_best_path_pins.py): enumeration of every alignment, the
 * bracket cost <= -ln p(l*) <= cost + ln(number of alignments), forced
 * alignments, planted alignments, and validity of the returned path.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ln(e^a + e^b) where an operand equal to -inf contributes nothing. */
static double log_add(double a, double b)
{
    if (a == -INFINITY) return b;
    if (b == -INFINITY) return a;
    double m = a > b ? a : b;
    return m + log(exp(a - m) + exp(b - m));
}

/*
 * One utterance.  x points at x[0, b, 0]; consecutive frames are `stride`
 * doubles apart.  grad (same addressing) may be NULL.  la / lb, if not NULL,
 * receive ln alpha and ln beta as [T_b][S] row-major.
 * Returns 0, or 1 if memory ran out.
 */
static int ctc_one(const double *x, long stride, int Tb, int A, int blank,
                   const int *label, int L, int Tfull,
                   double *cost, double *grad, double *la_out, double *lb_out)
{
    const int S = 2 * L + 1;
    int t, s, k;

    if (grad)
        for (t = 0; t < Tfull; ++t)
            for (k = 0; k < A; ++k) grad[t * stride + k] = 0.0;

    if (Tb == 0) {
        *cost = (L == 0) ? 0.0 : INFINITY;
        return 0;
    }

    double *lp = (double *)malloc(sizeof(double) * (size_t)Tb * A);
    double *la = (double *)malloc(sizeof(double) * (size_t)Tb * S);
    double *lb = (double *)malloc(sizeof(double) * (size_t)Tb * S);
    int *ext = (int *)malloc(sizeof(int) * (size_t)S);
    double *occ = (double *)malloc(sizeof(double) * (size_t)A);
    if (!lp || !la || !lb || !ext || !occ) {
        free(lp); free(la); free(lb); free(ext); free(occ);
        return 1;
    }

    /* blank-interleaved label: blank, l_0, blank, l_1, ..., l_{L-1}, blank */
    for (s = 0; s < S; ++s) ext[s] = (s % 2 == 0) ? blank : label[(s - 1) / 2];

    /* log-softmax of every valid frame */
    for (t = 0; t < Tb; ++t) {
        const double *row = x + t * stride;
        double mx = row[0], sum = 0.0;
        for (k = 1; k < A; ++k) if (row[k] > mx) mx = row[k];
        for (k = 0; k < A; ++k) sum += exp(row[k] - mx);
        double lse = mx + log(sum);
        for (k = 0; k < A; ++k) lp[(size_t)t * A + k] = row[k] - lse;
    }

    /* forward pass */
    for (s = 0; s < S; ++s) la[s] = -INFINITY;
    la[0] = lp[blank];
    if (S > 1) la[1] = lp[ext[1]];
    for (t = 1; t < Tb; ++t) {
        const double *prev = la + (size_t)(t - 1) * S;
        double *cur = la + (size_t)t * S;
        for (s = 0; s < S; ++s) {
            double acc = prev[s];
            if (s >= 1) acc = log_add(acc, prev[s - 1]);
            if (s >= 2 && ext[s] != blank && ext[s] != ext[s - 2])
                acc = log_add(acc, prev[s - 2]);
            cur[s] = (acc == -INFINITY) ? -INFINITY : acc + lp[(size_t)t * A + ext[s]];
        }
    }
    double lnp = la[(size_t)(Tb - 1) * S + S - 1];
    if (S > 1) lnp = log_add(lnp, la[(size_t)(Tb - 1) * S + S - 2]);

    /* backward pass, emission of the own frame left out */
    {
        double *last = lb + (size_t)(Tb - 1) * S;
        for (s = 0; s < S; ++s) last[s] = -INFINITY;
        last[S - 1] = 0.0;
        if (S > 1) last[S - 2] = 0.0;
    }
    for (t = Tb - 2; t >= 0; --t) {
        const double *next = lb + (size_t)(t + 1) * S;
        const double *lpn = lp + (size_t)(t + 1) * A;
        double *cur = lb + (size_t)t * S;
        for (s = 0; s < S; ++s) {
            double acc = (next[s] == -INFINITY) ? -INFINITY : next[s] + lpn[ext[s]];
            if (s + 1 < S && next[s + 1] != -INFINITY)
                acc = log_add(acc, next[s + 1] + lpn[ext[s + 1]]);
            if (s + 2 < S && ext[s] != blank && ext[s + 2] != ext[s] && next[s + 2] != -INFINITY)
                acc = log_add(acc, next[s + 2] + lpn[ext[s + 2]]);
            cur[s] = acc;
        }
    }

    if (la_out) memcpy(la_out, la, sizeof(double) * (size_t)Tb * S);
    if (lb_out) memcpy(lb_out, lb, sizeof(double) * (size_t)Tb * S);

    if (lnp == -INFINITY) {
        *cost = INFINITY;            /* no alignment exists; gradient stays zero */
    } else {
        *cost = -lnp;
        if (grad) {
            for (t = 0; t < Tb; ++t) {
                for (k = 0; k < A; ++k) occ[k] = 0.0;
                for (s = 0; s < S; ++s) {
                    double a = la[(size_t)t * S + s], b = lb[(size_t)t * S + s];
                    if (a == -INFINITY || b == -INFINITY) continue;
                    occ[ext[s]] += exp(a + b - lnp);
                }
                for (k = 0; k < A; ++k)
                    grad[t * stride + k] = exp(lp[(size_t)t * A + k]) - occ[k];
            }
        }
    }

    free(lp); free(la); free(lb); free(ext); free(occ);
    return 0;
}

/*
 * Batched entry point.
 *   x, grads      [T, B, A] doubles, A fastest (grads may be NULL)
 *   flat_labels   concatenation of the B label strings
 *   costs         [B]
 *   log_alpha/log_beta  NULL, or [B][T][s_pad] doubles: the first T_b x S_b block
 *                 of utterance b is filled row-major with pitch s_pad
 *   nthreads      OpenMP threads (<= 0: library default)
 * Returns 0 on success, 1 on allocation failure, 2 on invalid arguments.
 */
int ctc_oracle(const double *x, int T, int B, int A,
               const int *flat_labels, const int *label_lengths, const int *input_lengths,
               int blank, double *costs, double *grads,
               double *log_alpha, double *log_beta, int s_pad, int nthreads)
{
    if (T < 0 || B < 0 || A < 1 || blank < 0 || blank >= A) return 2;
    long *offs = (long *)malloc(sizeof(long) * (size_t)(B + 1));
    if (!offs) return 1;
    offs[0] = 0;
    for (int b = 0; b < B; ++b) {
        if (label_lengths[b] < 0 || input_lengths[b] < 0 || input_lengths[b] > T) { free(offs); return 2; }
        offs[b + 1] = offs[b] + label_lengths[b];
    }
    for (long i = 0; i < offs[B]; ++i)
        if (flat_labels[i] < 0 || flat_labels[i] >= A || flat_labels[i] == blank) { free(offs); return 2; }

    int failed = 0;
    const long stride = (long)B * A;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (int b = 0; b < B; ++b) {
        const int L = label_lengths[b], Tb = input_lengths[b], S = 2 * L + 1;
        double *la = NULL, *lb = NULL, *tmp_a = NULL, *tmp_b = NULL;
        if (log_alpha && Tb > 0) tmp_a = (double *)malloc(sizeof(double) * (size_t)Tb * S);
        if (log_beta && Tb > 0) tmp_b = (double *)malloc(sizeof(double) * (size_t)Tb * S);
        la = tmp_a; lb = tmp_b;
        int rc = ctc_one(x + (long)b * A, stride, Tb, A, blank, flat_labels + offs[b], L, T,
                         &costs[b], grads ? grads + (long)b * A : NULL, la, lb);
        if (rc) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
        for (int t = 0; t < Tb && !rc; ++t) {
            if (tmp_a) memcpy(log_alpha + ((size_t)b * T + t) * s_pad, tmp_a + (size_t)t * S, sizeof(double) * S);
            if (tmp_b) memcpy(log_beta + ((size_t)b * T + t) * s_pad, tmp_b + (size_t)t * S, sizeof(double) * S);
        }
        free(tmp_a); free(tmp_b);
    }
    free(offs);
    return failed;
}

/* Threads the batched entry point uses when nthreads <= 0. */
int ctc_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Most probable alignment of one utterance (max-product over the same lattice).
 * states[t] receives the lattice state of frame t (0-based index into the
 * blank-interleaved label: even = blank, odd s = label[(s-1)/2]) for t < Tb and
 * -1 for Tb <= t < Tfull.  *score = -ln of that alignment's probability, +inf
 * (and all states -1) when no alignment exists.  Among equally good
 * predecessors the one with the highest state index wins; callers must not
 * rely on that.
 */
static int best_path_one(const double *x, long stride, int Tb, int A, int blank,
                         const int *label, int L, int Tfull, double *score, int *states)
{
    const int S = 2 * L + 1;
    int t, s, k;
    for (t = 0; t < Tfull; ++t) states[t] = -1;
    if (Tb == 0) {
        *score = (L == 0) ? 0.0 : INFINITY;
        return 0;
    }
    double *lp = (double *)malloc(sizeof(double) * (size_t)Tb * A);
    double *v = (double *)malloc(sizeof(double) * (size_t)Tb * S);
    int *from = (int *)malloc(sizeof(int) * (size_t)Tb * S);
    int *ext = (int *)malloc(sizeof(int) * (size_t)S);
    if (!lp || !v || !from || !ext) {
        free(lp); free(v); free(from); free(ext);
        return 1;
    }
    for (s = 0; s < S; ++s) ext[s] = (s % 2 == 0) ? blank : label[(s - 1) / 2];
    for (t = 0; t < Tb; ++t) {
        const double *row = x + t * stride;
        double mx = row[0], sum = 0.0;
        for (k = 1; k < A; ++k) if (row[k] > mx) mx = row[k];
        for (k = 0; k < A; ++k) sum += exp(row[k] - mx);
        double lse = mx + log(sum);
        for (k = 0; k < A; ++k) lp[(size_t)t * A + k] = row[k] - lse;
    }
    for (s = 0; s < S; ++s) { v[s] = -INFINITY; from[s] = -1; }
    v[0] = lp[blank];
    if (S > 1) v[1] = lp[ext[1]];
    for (t = 1; t < Tb; ++t) {
        const double *prev = v + (size_t)(t - 1) * S;
        for (s = 0; s < S; ++s) {
            double best = prev[s];
            int arg = s;
            if (s >= 1 && prev[s - 1] >= best) { best = prev[s - 1]; arg = s - 1; }
            if (s >= 2 && ext[s] != blank && ext[s] != ext[s - 2] && prev[s - 2] >= best) {
                best = prev[s - 2];
                arg = s - 2;
            }
            if (best == -INFINITY) {
                v[(size_t)t * S + s] = -INFINITY;
                from[(size_t)t * S + s] = -1;
            } else {
                v[(size_t)t * S + s] = best + lp[(size_t)t * A + ext[s]];
                from[(size_t)t * S + s] = arg;
            }
        }
    }
    const double *last = v + (size_t)(Tb - 1) * S;
    int end = S - 1;
    if (S > 1 && last[S - 2] > last[S - 1]) end = S - 2;
    if (last[end] == -INFINITY) {
        *score = INFINITY;
    } else {
        *score = -last[end];
        s = end;
        for (t = Tb - 1; t >= 0; --t) {
            states[t] = s;
            s = from[(size_t)t * S + s];
        }
    }
    free(lp); free(v); free(from); free(ext);
    return 0;
}

/*
 * Batched most probable alignment.
 *   x            [T, B, A] doubles, A fastest
 *   scores       [B]
 *   states       [B][T] ints (utterance-major)
 * Return codes as ctc_oracle.
 */
int ctc_oracle_best_path(const double *x, int T, int B, int A,
                         const int *flat_labels, const int *label_lengths, const int *input_lengths,
                         int blank, double *scores, int *states, int nthreads)
{
    if (T < 0 || B < 0 || A < 1 || blank < 0 || blank >= A) return 2;
    long *offs = (long *)malloc(sizeof(long) * (size_t)(B + 1));
    if (!offs) return 1;
    offs[0] = 0;
    for (int b = 0; b < B; ++b) {
        if (label_lengths[b] < 0 || input_lengths[b] < 0 || input_lengths[b] > T) { free(offs); return 2; }
        offs[b + 1] = offs[b] + label_lengths[b];
    }
    for (long i = 0; i < offs[B]; ++i)
        if (flat_labels[i] < 0 || flat_labels[i] >= A || flat_labels[i] == blank) { free(offs); return 2; }
    int failed = 0;
    const long stride = (long)B * A;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (int b = 0; b < B; ++b) {
        int rc = best_path_one(x + (long)b * A, stride, input_lengths[b], A, blank,
                               flat_labels + offs[b], label_lengths[b], T, &scores[b],
                               states + (size_t)b * T);
        if (rc) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
    }
    free(offs);
    return failed;
}
