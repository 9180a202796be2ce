/*
 * CPU oracle for the SSM-layer prefill with cached-state resume and state
 * checkpoints.  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the
 * benchmark's CPU-baseline leg call it; the GPU library never does, and the
 * two share no code.
 *
 * What it computes is the definition itself, one token at a time, in double
 * precision, with no chunking, blocking or reordering:
 *
 *   The paper describes the SSM layer in words (Section 2.1; Section 3, "SSM
 *   State Properties"): a constant-size recurrent state is overwritten in
 *   place by every token.  Written out for a Mamba2-style layer with a scalar
 *   decay rate A[h] per head, for head h, channel p, state index n and the
 *   sequence-local token t = 1..len:
 *
 *       a_t      = exp(dt[t,h] * A[h])
 *       S_t[p,n] = a_t * S_{t-1}[p,n] + dt[t,h] * x[t,h,p] * B[t,g(h),n]
 *       y[t,h,p] = sum_n C[t,g(h),n] * S_t[p,n] + D[h] * x[t,h,p]
 *
 *   with g(h) = h / (H/G) (heads of a group are contiguous) and
 *   S_0 = the cached state of the matched prefix, or zero (Section 2.2:
 *   on a hit the prefix state is fetched before prefill; Section 4.1,
 *   two-pass prefill: the second pass starts from the prefix state).
 *
 *   A checkpoint at position p of a sequence (1 <= p <= len) is S_p, the state
 *   after exactly p tokens of that sequence (Section 4.1, "Obtaining states
 *   during prefill": the exact-position state, not the chunk-boundary one).
 *
 * Pins (tests/test_oracle_pins.py): unrolled closed-form sums by independent
 * O(T^2) loops, the A = 0 / B = 0 / dt = 0 / constant-input special cases
 * against numpy matmul and the geometric series, the prefix-cache invariant
 * at the paper's (80, 20) split, superposition, packing independence and
 * off-by-one sensitivity of checkpoints.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Scan one (sequence, head) pair.  S is a caller-provided [P*N] scratch. */
static void scan_one(int64_t t0, int64_t len, int h, int H, int P, int N, int G,
                     const float *x, const float *dt, const float *A,
                     const float *B, const float *C, const float *D,
                     const double *init,          /* [H,P,N] or NULL */
                     const int32_t *ckpt, int n_ckpt, int64_t slot0,
                     double *y_out, double *state_out, double *S)
{
    const int g = h / (H / G);
    const size_t PN = (size_t)P * (size_t)N;
    if (init)
        memcpy(S, init + (size_t)h * PN, PN * sizeof(double));
    else
        memset(S, 0, PN * sizeof(double));

    int next = 0; /* next checkpoint of this sequence, ascending */
    const double Ah = (double)A[h];
    const double Dh = (double)D[h];
    for (int64_t i = 0; i < len; ++i) {
        const int64_t t = t0 + i;
        const double dth = (double)dt[t * H + h];
        const double a = exp(dth * Ah);
        const float *xt = x + ((size_t)t * H + h) * P;
        const float *Bt = B + ((size_t)t * G + g) * N;
        const float *Ct = C + ((size_t)t * G + g) * N;
        double *yt = y_out ? y_out + ((size_t)t * H + h) * P : NULL;
        for (int p = 0; p < P; ++p) {
            const double xp = (double)xt[p];
            const double u = dth * xp;
            double *Sp = S + (size_t)p * N;
            double acc = 0.0;
            for (int n = 0; n < N; ++n) {
                const double s = a * Sp[n] + u * (double)Bt[n];
                Sp[n] = s;
                acc += (double)Ct[n] * s;
            }
            if (yt)
                yt[p] = acc + Dh * xp;
        }
        /* sequence-local token count after this token is i + 1 */
        while (next < n_ckpt && (int64_t)ckpt[next] == i + 1) {
            double *dst = state_out + ((size_t)(slot0 + next) * H + h) * PN;
            memcpy(dst, S, PN * sizeof(double));
            ++next;
        }
    }
}

/*
 * All pointers are host pointers.  Layouts (row-major, last index fastest):
 *   x [T,H,P], dt [T,H], A [H], B [T,G,N], C [T,G,N], D [H]      (float)
 *   cu_seqlens [batch+1], cu_ckpt [batch+1] (CSR into ckpt_pos), ckpt_pos
 *   init_state: array of `batch` pointers to double [H,P,N]; the array or
 *               any entry may be NULL (zero state)
 *   y_out [T,H,P] double (may be NULL), state_out [n_ckpt,H,P,N] double
 * Returns 0, or a negative value for malformed arguments.
 */
int oracle_ssm_prefill(int64_t T, int H, int P, int N, int G,
                       const float *x, const float *dt, const float *A,
                       const float *B, const float *C, const float *D,
                       int batch, const int32_t *cu_seqlens,
                       const double *const *init_state,
                       const int32_t *cu_ckpt, const int32_t *ckpt_pos,
                       double *y_out, double *state_out, int nthreads)
{
    if (H <= 0 || P <= 0 || N <= 0 || G <= 0 || H % G != 0 || batch < 0)
        return -1;
    if (!cu_seqlens || cu_seqlens[0] != 0 || (int64_t)cu_seqlens[batch] != T)
        return -2;
    for (int s = 0; s < batch; ++s) {
        const int64_t len = (int64_t)cu_seqlens[s + 1] - cu_seqlens[s];
        if (len < 0)
            return -2;
        const int c0 = cu_ckpt ? cu_ckpt[s] : 0, c1 = cu_ckpt ? cu_ckpt[s + 1] : 0;
        for (int k = c0; k < c1; ++k) {
            if (ckpt_pos[k] < 1 || ckpt_pos[k] > len)
                return -3;
            if (k > c0 && ckpt_pos[k] <= ckpt_pos[k - 1])
                return -3;
        }
    }
    if (nthreads < 1)
        nthreads = 1;
    const size_t PN = (size_t)P * (size_t)N;
    const int64_t work = (int64_t)batch * H;
    int failed = 0;
#pragma omp parallel num_threads(nthreads)
    {
        double *S = (double *)malloc(PN * sizeof(double));
        if (!S) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t w = 0; w < work; ++w) {
            if (!S)
                continue;
            const int s = (int)(w / H), h = (int)(w % H);
            const int64_t t0 = cu_seqlens[s];
            const int64_t len = (int64_t)cu_seqlens[s + 1] - t0;
            const int c0 = cu_ckpt ? cu_ckpt[s] : 0, c1 = cu_ckpt ? cu_ckpt[s + 1] : 0;
            const double *init = init_state ? init_state[s] : NULL;
            scan_one(t0, len, h, H, P, N, G, x, dt, A, B, C, D, init,
                     ckpt_pos ? ckpt_pos + c0 : NULL, c1 - c0, c0, y_out, state_out, S);
        }
        free(S);
    }
    return failed ? -4 : 0;
}

/* Number of threads the parallel region would really get. */
int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
