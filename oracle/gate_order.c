/* TEST INFRASTRUCTURE ONLY - part of the CPU oracle; the product path never links or calls this.
 *
 * Gate projection of the padding-free MoE layer (the "FFN(tokens)" inside the gating function of the
 * paper's Listing 1, described in Appendix B.3 as the projection of [S,H] tokens to [S,E] logits),
 * evaluated in single precision in ONE fixed summation order, so that the top-k decision taken on these
 * logits is reproducible bit for bit by any implementation that follows the same order.
 *
 * The order (a reading this build adds; the paper does not fix one):
 *   partial[l] (l = 0..63) starts at +0.0f and absorbs, for i = l, l+64, l+128, ... in ascending i,
 *       partial[l] = fmaf(x[t,i], w[i,e], partial[l])            (one rounding per term)
 *   the 64 partials are folded by halving: for off = 32,16,8,4,2,1:  partial[l] += partial[l+off], l < off
 *   logits[t,e] = partial[0] + bias[e]   (bias omitted when NULL)
 *
 * Plain C, one (t,e) pair at a time, nothing blocked or reordered.
 */
#include <math.h>
#include <stddef.h>

void xmoe_oracle_gate_logits_f32(const float* x, const float* w, const float* bias, float* logits,
                                 int T, int d, int E) {
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            float partial[64];
            for (int l = 0; l < 64; ++l) partial[l] = 0.0f;
            for (int i = 0; i < d; ++i) {
                int l = i % 64;
                partial[l] = fmaf(x[(size_t)t * d + i], w[(size_t)i * E + e], partial[l]);
            }
            for (int off = 32; off >= 1; off /= 2)
                for (int l = 0; l < off; ++l) partial[l] = partial[l] + partial[l + off];
            float v = partial[0];
            if (bias) v = v + bias[e];
            logits[(size_t)t * E + e] = v;
        }
    }
}
