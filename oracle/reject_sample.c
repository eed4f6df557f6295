/*
 * CPU oracle for the lossless rejection-sampling pass of the speculative-decoding
 * verify step.  TEST INFRASTRUCTURE ONLY: nothing on the product path may include,
 * link or call this file.  It shares no code with the HIP kernels.
 *
 * What it follows.  The paper (Introduction, paragraph on speculative decoding; Section 2.1)
 * only states that the target model verifies the drafted tokens "through a rejection
 * procedure that preserves its output distribution" and cites the standard procedure:
 * a draft token x drawn from q is kept with probability min(1, p(x)/q(x)); at the first
 * rejection a replacement is drawn from norm(max(0, p - q)); if all k drafts are kept a
 * bonus token is drawn from the next target distribution.  The acceptance length the
 * paper reports (Section 2.2) counts every token produced by a step, so it is n + 1.
 *
 * The mapping uniforms -> tokens is a convention of this build (the paper fixes only the
 * output distribution):
 *   - random numbers come from Philox4x32-10 (Salmon et al., SC'11), key = (seed_lo, seed_hi),
 *     counter = (c0, row, b, step*4 + stream);
 *   - stream 0, c0 = 0, word 0: the accept uniform  u = (r >> 8) * 2^-24   in [0,1);
 *   - stream 1, c0 = v >> 2, word v & 3: the per-vocabulary uniform
 *         u_v = ((r >> 9) + 0.5) * 2^-23   in (0,1), exactly representable in fp32;
 *   - accept test: u * Q < P, strict, in fp64 (P >= Q > 0 always accepts, P == 0 never);
 *   - categorical draw by exponential race (equivalent to Gumbel-max):
 *         y = argmax_v  w_v / (-ln u_v)   over w_v > 0, ties to the lowest v,
 *     which does not depend on the order in which the vocabulary is scanned.
 * Everything is computed in fp64 from the fp32 inputs, one element at a time, in index order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

static void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(prod1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prod1;
        uint32_t n2 = (uint32_t)(prod0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prod0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Raw generator, exported so that tests can pin it against published known answers. */
void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out)
{
    philox4x32_10(ctr, key, out);
}

static uint32_t draw_word(uint64_t seed, uint64_t step, int stream, uint32_t c0, int row, int b, int word)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4] = { c0, (uint32_t)row, (uint32_t)b, (uint32_t)(step * 4u + (uint64_t)stream) };
    uint32_t out[4];
    philox4x32_10(ctr, key, out);
    return out[word];
}

double oracle_uniform_accept(uint64_t seed, uint64_t step, int b, int row)
{
    uint32_t r = draw_word(seed, step, 0, 0u, row, b, 0);
    return (double)(r >> 8) * (1.0 / 16777216.0);
}

double oracle_uniform_vocab(uint64_t seed, uint64_t step, int b, int row, int v)
{
    uint32_t r = draw_word(seed, step, 1, (uint32_t)v >> 2, row, b, v & 3);
    return ((double)(r >> 9) + 0.5) * (1.0 / 8388608.0);
}

/* p[v] = softmax(logits[v] / T) in fp64 with the maximum subtracted first. */
static void softmax_row(const float* logits, int V, double T, double* p)
{
    double m = -INFINITY;
    for (int v = 0; v < V; ++v) {
        double z = (double)logits[v] / T;
        if (z > m) m = z;
    }
    double S = 0.0;
    for (int v = 0; v < V; ++v) {
        p[v] = exp((double)logits[v] / T - m);
        S += p[v];
    }
    for (int v = 0; v < V; ++v) p[v] /= S;
}

/*
 * logits [B, k+1, V] fp32: row i is the target's distribution of the token that follows
 *                          input position i (row i judges draft i+1; row k is the bonus row).
 * q      [B, k, V]   fp32 probabilities the drafts were sampled from.
 * draft  [B, k]      int32 drafted tokens.
 * accept_len [B]     out: n in 0..k.
 * out_tokens [B,k+1] out: the n kept drafts, then the resampled/bonus token, then -1.
 * dbg_pqu [B, k, 3]  out, may be NULL: P, Q, u of every accept test that was evaluated, NaN elsewhere.
 * dbg_keys [B, 2]    out, may be NULL: the winning key and the runner-up key of the draw.
 * Returns 0, or -1 on invalid arguments.
 */
int oracle_reject_sample(int B, int k, int V, const float* logits, const float* q, const int32_t* draft,
                         float temperature, uint64_t seed, uint64_t step,
                         int32_t* accept_len, int32_t* out_tokens, double* dbg_pqu, double* dbg_keys)
{
    if (B < 0 || k < 0 || V <= 0 || !(temperature > 0.0f)) return -1;
    double T = (double)temperature;
    double* p = (double*)malloc(sizeof(double) * (size_t)V);
    double* w = (double*)malloc(sizeof(double) * (size_t)V);
    if (!p || !w) { free(p); free(w); return -1; }

    for (int b = 0; b < B; ++b) {
        const float* L = logits + (size_t)b * (size_t)(k + 1) * (size_t)V;
        const float* Qb = q + (size_t)b * (size_t)k * (size_t)V;
        if (dbg_pqu)
            for (int j = 0; j < 3 * k; ++j) dbg_pqu[(size_t)b * 3 * k + j] = NAN;

        int n = 0;
        for (int i = 0; i < k; ++i) {
            int x = draft[(size_t)b * k + i];
            if (x < 0 || x >= V) { free(p); free(w); return -1; }
            softmax_row(L + (size_t)i * V, V, T, p);
            double P = p[x];
            double Q = (double)Qb[(size_t)i * V + x];
            double u = oracle_uniform_accept(seed, step, b, i);
            if (dbg_pqu) {
                double* d = dbg_pqu + ((size_t)b * k + i) * 3;
                d[0] = P; d[1] = Q; d[2] = u;
            }
            if (u * Q < P) n += 1; else break;
        }

        /* weights of the final draw: residual at the first rejection, target itself for the bonus */
        softmax_row(L + (size_t)n * V, V, T, p);
        int any = 0;
        if (n < k) {
            for (int v = 0; v < V; ++v) {
                double r = p[v] - (double)Qb[(size_t)n * V + v];
                w[v] = r > 0.0 ? r : 0.0;
                if (w[v] > 0.0) any = 1;
            }
        }
        if (!any)                       /* bonus row, or a residual that is identically zero */
            for (int v = 0; v < V; ++v) w[v] = p[v];

        int y = -1;
        double best = -1.0, second = -1.0;
        for (int v = 0; v < V; ++v) {
            if (!(w[v] > 0.0)) continue;
            double e = -log(oracle_uniform_vocab(seed, step, b, n, v));
            double key = w[v] / e;
            if (key > best) { second = best; best = key; y = v; }
            else if (key > second) second = key;
        }
        if (dbg_keys) { dbg_keys[2 * b] = best; dbg_keys[2 * b + 1] = second; }

        accept_len[b] = n;
        int32_t* o = out_tokens + (size_t)b * (k + 1);
        for (int i = 0; i < n; ++i) o[i] = draft[(size_t)b * k + i];
        o[n] = y;
        for (int i = n + 1; i <= k; ++i) o[i] = -1;
    }
    free(p); free(w);
    return 0;
}

/* Per-vocabulary uniform of the draft model's own draw: stream 2, row = index of the draft position. */
double oracle_uniform_draft(uint64_t seed, uint64_t step, int b, int row, int v)
{
    uint32_t r = draw_word(seed, step, 2, (uint32_t)v >> 2, row, b, v & 3);
    return ((double)(r >> 9) + 0.5) * (1.0 / 8388608.0);
}

/*
 * The draft side of a speculation step (Section 2.1: "a draft model proposes several tokens"):
 * the proposal distribution of draft position `row` and one token drawn from it.
 *   logits [B, V] fp32: the draft model's logits for that position.
 *   q_out  [B, V] fp32: q = softmax(logits / T), the distribution the verifier is later given.
 *   tokens [B]    int32: x ~ q by the same exponential race as above, on stream 2:
 *                        x = argmax_v q_v / (-ln u_v), ties to the lowest v.
 *   dbg_keys [B, 2] may be NULL: winning and runner-up key.
 * Convention of this build; the paper fixes only that x is a sample of q.
 */
int oracle_draft_sample(int B, int V, const float* logits, float temperature, uint64_t seed, uint64_t step, int row,
                        int32_t* tokens, float* q_out, double* dbg_keys)
{
    if (B < 0 || V <= 0 || row < 0 || !(temperature > 0.0f)) return -1;
    double* p = (double*)malloc(sizeof(double) * (size_t)V);
    if (!p) return -1;
    for (int b = 0; b < B; ++b) {
        softmax_row(logits + (size_t)b * V, V, (double)temperature, p);
        int x = -1;
        double best = -1.0, second = -1.0;
        for (int v = 0; v < V; ++v) {
            q_out[(size_t)b * V + v] = (float)p[v];
            if (!(p[v] > 0.0)) continue;
            double key = p[v] / -log(oracle_uniform_draft(seed, step, b, row, v));
            if (key > best) { second = best; best = key; x = v; }
            else if (key > second) second = key;
        }
        tokens[b] = x;
        if (dbg_keys) { dbg_keys[2 * b] = best; dbg_keys[2 * b + 1] = second; }
    }
    free(p);
    return 0;
}
