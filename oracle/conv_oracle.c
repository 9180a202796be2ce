/*
 * CPU oracle for the causal depthwise convolution that precedes the SSM scan
 * in a Mamba2-style layer, with cached-state resume and state checkpoints.
 * TEST INFRASTRUCTURE ONLY, like ssm_oracle.c; shares no code with the GPU
 * library.
 *
 * The paper names this block only through its state (Appendix A.1, "Memory
 * footprint": every SSM layer carries a conv_1d state of
 * in_channels * conv_kernel elements, 6.1 % of a cache entry, which is part
 * of every cached prefix).  The operation itself is the textbook one, written
 * out here for channel c, kernel width K and the sequence-local token
 * t = 1..len:
 *
 *     out[t,c] = act( bias[c] + sum_{j=0}^{K-1} w[c,j] * z[t-K+1+j, c] )
 *
 * where z[i,c] = in[i,c] for i >= 1 and, for i <= 0, the inputs that preceded
 * the sequence: z[0] is the newest and z[-(K-2)] the oldest of the cached
 * prefix's last K-1 inputs, or zero without a cached prefix.  w[c,K-1]
 * multiplies the current token.  act is the identity or SiLU,
 * v / (1 + exp(-v)).
 *
 * Cached state.  The state after p tokens holds the last K inputs of channel
 * c, oldest first: state[c][m] = z[p-K+1+m, c], m = 0..K-1 (the paper's size
 * of conv_kernel elements per channel).  A resumed call uses its last K-1
 * entries as the inputs that preceded the sequence; entry 0 is carried only to
 * keep the cached layout.
 *
 * All arithmetic in double, in the order written; no blocking.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

/* value of z[i] (i sequence-local, 1-based for real tokens) of channel c */
static double z_at(int64_t i, int64_t t0, int c, int Cch, int K, const float *in, const double *init)
{
    if (i >= 1)
        return (double)in[(size_t)(t0 + i - 1) * Cch + c];
    /* i = 0 is init[c][K-1], i = -(K-2) is init[c][1] */
    if (!init)
        return 0.0;
    return init[(size_t)c * K + (K - 1 + i)];
}

/*
 * in [T,Cch] fp32, w [Cch,K], bias [Cch] or NULL, cu_seqlens [batch+1],
 * init_state: NULL or [batch] pointers (NULL entry = zeros) to double [Cch,K],
 * cu_ckpt/ckpt_pos as in oracle_ssm_prefill, act: 0 identity, 1 SiLU.
 * out [T,Cch] double (may be NULL), state_out [n_ckpt,Cch,K] double.
 * Returns 0, or a negative code for malformed arguments.
 */
int oracle_conv1d_prefill(int64_t T, int Cch, int K, const float *in, const float *w, const float *bias,
                          int batch, const int32_t *cu_seqlens, const double *const *init_state,
                          const int32_t *cu_ckpt, const int32_t *ckpt_pos, int act,
                          double *out, double *state_out)
{
    if (T < 0 || Cch <= 0 || K < 1 || batch < 0 || !cu_seqlens || cu_seqlens[0] != 0 || cu_seqlens[batch] != T)
        return -1;
    for (int s = 0; s < batch; ++s) {
        const int64_t t0 = cu_seqlens[s], len = cu_seqlens[s + 1] - t0;
        if (len < 0)
            return -2;
        const double *init = init_state ? init_state[s] : NULL;
        for (int64_t t = 1; t <= len; ++t)
            for (int c = 0; c < Cch; ++c) {
                double v = bias ? (double)bias[c] : 0.0;
                for (int j = 0; j < K; ++j)
                    v += (double)w[(size_t)c * K + j] * z_at(t - K + 1 + j, t0, c, Cch, K, in, init);
                if (act == 1)
                    v = v / (1.0 + exp(-v));
                if (out)
                    out[(size_t)(t0 + t - 1) * Cch + c] = v;
            }
        if (cu_ckpt)
            for (int32_t k = cu_ckpt[s]; k < cu_ckpt[s + 1]; ++k) {
                const int64_t p = ckpt_pos[k];
                if (p < 1 || p > len || (k > cu_ckpt[s] && p <= ckpt_pos[k - 1]))
                    return -3;
                for (int c = 0; c < Cch; ++c)
                    for (int m = 0; m < K; ++m) {
                        /* p >= 1, so the index is at least -(K-2): never older than what a resume keeps */
                        const double val = z_at(p - K + 1 + m, t0, c, Cch, K, in, init);
                        state_out[((size_t)k * Cch + c) * K + m] = val;
                    }
            }
    }
    return 0;
}
