/*
 * CPU oracle for the projection that turns dense 3x3 weights into PCONV form.  TEST
 * INFRASTRUCTURE ONLY; nothing in the product path may call into this file, and it shares no code
 * with the library.
 *
 * The paper ("Accuracy Analysis") produces its models with an ADMM pruner extended to the two
 * PCONV constraints - every kernel carries the taps of one Sparse Convolution Pattern from the
 * table (pattern pruning), and only a given number of kernels survive (connectivity pruning) - and
 * leaves the details to supplemental material that is not available.  What an ADMM pruner needs
 * from such a constraint set is the Euclidean projection onto it, and that has a plain definition:
 * among all weight tensors Z that satisfy both constraints, the one closest to W in the sum of
 * squared differences.  Because the constraints act per kernel, the minimiser is found directly:
 *
 *   e[f,c,p] = sum over the taps t of mask p of W[f,c,t]^2        energy a kernel keeps under pattern p
 *   pid[f,c] = the p with the largest e[f,c,p]                    (smallest p among equals)
 *   keep the `keep` kernels with the largest e[f,c,pid[f,c]]      (smallest f*C + c among equals)
 *
 * since dropping kernel (f,c) costs its whole energy, keeping it under pattern p costs the energy
 * outside the mask, and the saving e[f,c,p] of keeping is what the two choices maximise.
 * Arithmetic: squares and sums in double, taps in ascending order (the square of a float is exact
 * in double; a decision between two sums is therefore taken on correctly ordered values except for
 * ties in the last bit of a nine-term double sum, which both sides resolve the same way by using
 * this same order).
 *
 * Parity status: pinned by tests/test_oracle_project.py against exhaustive search over every
 * assignment on tiny layers, and against closed special cases (one dense mask = largest kernels by
 * norm; keep all; keep none).  Parity with the paper's own models is unpinned: the paper prints
 * no assignment and its algorithm text is in the missing supplement.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct { double e; int idx; } orc_kernel_energy;

static int by_energy_desc(const void *a, const void *b)
{
    const orc_kernel_energy *x = (const orc_kernel_energy *)a, *y = (const orc_kernel_energy *)b;
    if (x->e != y->e) return x->e > y->e ? -1 : 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx ? 1 : 0);
}

/* w [F][C][3][3]; table [np] 9-bit masks; keep = number of kernels that survive (0 .. F*C).
 * Out: pattern_id [F][C] (for every kernel, kept or not), conn [F][C] (1 = kept). */
void orc_project(const float *w, const uint16_t *table, int np, int f_count, int c_count, long keep,
                 uint8_t *pattern_id, uint8_t *conn)
{
    const long total = (long)f_count * c_count;
    orc_kernel_energy *ke = (orc_kernel_energy *)malloc((size_t)(total > 0 ? total : 1) * sizeof(orc_kernel_energy));
    for (long k = 0; k < total; ++k) {
        const float *kw = w + 9 * k;
        double best = -1.0;
        int best_p = 0;
        for (int p = 0; p < np; ++p) {
            double e = 0.0;
            for (int t = 0; t < 9; ++t)
                if ((table[p] >> t) & 1) e += (double)kw[t] * (double)kw[t];
            if (e > best) { best = e; best_p = p; }
        }
        pattern_id[k] = (uint8_t)best_p;
        ke[k].e = best;
        ke[k].idx = (int)k;
        conn[k] = 0;
    }
    qsort(ke, (size_t)total, sizeof(orc_kernel_energy), by_energy_desc);
    for (long i = 0; i < keep && i < total; ++i) conn[ke[i].idx] = 1;
    free(ke);
}
