/*
 * CPU oracle for the parameter-server hot path of "Training Through Failure"
 * (arxiv 2406.05546).  TEST INFRASTRUCTURE ONLY: plain, slow, fp64, direct
 * loops.  Nothing in the product path may call into this file; it shares no
 * code with the HIP kernels.
 *
 * What it computes
 *   - the gradient of one worker's mean minibatch loss for the small CNN of
 *     the paper's model endnote (conv 3x3 -> ReLU -> maxpool 2x2, twice; FC;
 *     ReLU; dropout; FC; softmax cross-entropy), by the chain rule through
 *     exactly those operations (Section 3.3, worker step: gradients are
 *     generated from one weight snapshot on one minibatch);
 *   - the dropout keep-mask from the Philox4x32-10 counter-based generator
 *     (Salmon, Moraes, Dror, Shaw, SC'11), keyed by (seed, minibatch, sample,
 *     unit).
 * The three server update rules (Section 2.1 sync/async, Section 3.3
 * stateless) are one-liners and live in oracle.py.
 *
 * Layer sizes are run-time parameters so that the same code is checked by
 * finite differences on tiny nets and then used at the paper's sizes.
 *
 * Flat parameter vector (floats, in this order):
 *   conv1.W[C1][1][3][3], conv1.b[C1], conv2.W[C2][C1][3][3], conv2.b[C2],
 *   fc1.W[F][C2*(H/4)*(W/4)] (input index = c*(H/4)*(W/4) + y*(W/4) + x),
 *   fc1.b[F], fc2.W[NC][F], fc2.b[NC].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t H, W;   /* input image, one channel; both divisible by 4 */
    int32_t C1, C2; /* conv1 / conv2 output channels */
    int32_t F;      /* fc1 units */
    int32_t NC;     /* classes */
} oracle_dims;

int64_t oracle_param_count(const oracle_dims* d)
{
    int64_t feat = (int64_t)d->C2 * (d->H / 4) * (d->W / 4);
    return (int64_t)d->C1 * 9 + d->C1 + (int64_t)d->C2 * d->C1 * 9 + d->C2 + (int64_t)d->F * feat + d->F +
           (int64_t)d->NC * d->F + d->NC;
}

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon et al. 2011): 10 rounds; each round multiplies
 * counter words 0 and 2 by two fixed odd constants, swaps high/low halves
 * into place and xors in the key; the key is advanced by two Weyl
 * constants between rounds.                                           */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        if (r > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Dropout keep mask for one minibatch.  Unit u of sample s takes word (u % 4)
 * of Philox(counter = {mb_lo, mb_hi, s, u / 4}, key = {seed_lo, seed_hi});
 * the unit is dropped iff that word is below `threshold` = floor(p * 2^32).
 * keep[s*F + u] = 1 if kept.                                            */
void oracle_dropout_keep(uint64_t seed, uint64_t minibatch_id, int32_t B, int32_t F, uint32_t threshold,
                         uint8_t* keep)
{
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int32_t s = 0; s < B; ++s)
        for (int32_t u = 0; u < F; ++u) {
            uint32_t ctr[4] = {(uint32_t)minibatch_id, (uint32_t)(minibatch_id >> 32), (uint32_t)s,
                               (uint32_t)(u / 4)};
            uint32_t w[4];
            oracle_philox4x32_10(ctr, key, w);
            keep[(int64_t)s * F + u] = (w[u % 4] >= threshold) ? 1 : 0;
        }
}

/* ------------------------------------------------------------------ */
/* conv 3x3, pad 1, stride 1, correlation (no kernel flip), plus bias.
 * in [Cin][H][W], Wt [Cout][Cin][3][3], out [Cout][H][W] (pre-activation). */
static void conv3x3(int Cin, int Cout, int H, int W, const double* in, const double* Wt, const double* b,
                    double* out)
{
    for (int o = 0; o < Cout; ++o)
        for (int y = 0; y < H; ++y)
            for (int x = 0; x < W; ++x) {
                double acc = b[o];
                for (int c = 0; c < Cin; ++c)
                    for (int dy = 0; dy < 3; ++dy)
                        for (int dx = 0; dx < 3; ++dx) {
                            int yy = y + dy - 1, xx = x + dx - 1;
                            if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                            acc += Wt[((o * Cin + c) * 3 + dy) * 3 + dx] * in[(c * H + yy) * W + xx];
                        }
                out[(o * H + y) * W + x] = acc;
            }
}

/* ReLU then 2x2 stride-2 max pool.  Because max and ReLU commute, the window
 * winner is chosen on the pre-activation: scan (0,0),(0,1),(1,0),(1,1), a
 * later element replaces the current best only if strictly greater.  code =
 * dy*2+dx of the winner; top = its pre-activation value; margin = top minus
 * the best of the other three.  pooled = max(top, 0).                   */
static void relu_pool2(int C, int H, int W, const double* pre, double* pooled, uint8_t* code, double* top,
                       double* margin)
{
    int Hp = H / 2, Wp = W / 2;
    for (int c = 0; c < C; ++c)
        for (int py = 0; py < Hp; ++py)
            for (int px = 0; px < Wp; ++px) {
                double best = 0.0, second = -INFINITY;
                int bi = -1;
                for (int k = 0; k < 4; ++k) {
                    double v = pre[(c * H + 2 * py + k / 2) * W + 2 * px + k % 2];
                    if (bi < 0) {
                        best = v; bi = 0;
                    } else if (v > best) {
                        second = best; best = v; bi = k;
                    } else if (v > second) {
                        second = v;
                    }
                }
                int idx = (c * Hp + py) * Wp + px;
                pooled[idx] = best > 0.0 ? best : 0.0;
                code[idx] = (uint8_t)bi;
                top[idx] = best;
                margin[idx] = best - second;
            }
}

/* Gradient of one worker's MEAN minibatch loss w.r.t. the flat parameter
 * vector, evaluated at `theta` (the worker's weight snapshot, which may be
 * stale: Section 2.1 async rule, Section 2.3 outage rule).
 *
 *  x     [B][H*W]   pixels
 *  y     [B]        labels
 *  keep  [B][F]     dropout keep mask (1 = kept); kept units are scaled by
 *                   `scale` (= 1/(1-p)), forward and backward
 *  grad  [P]        out
 *  loss  [1]        out, mean cross-entropy (natural log)
 * Optional per-sample records (NULL to skip), used for decision parity:
 *  code1/top1/margin1 [B][C1*(H/2)*(W/2)], code2/top2/margin2 [B][C2*(H/4)*(W/4)],
 *  hpre [B][F] fc1 pre-activation, z [B][NC] logits.
 * Optional forced decisions: n_forced records of four int32 {sample, layer, index, value}.  A max
 * or a ReLU whose arguments tie within rounding reach has two equally valid outcomes; a record
 * makes this pass take the stated one: layer 1 / 2 = pooled output `index` of pool1 / pool2 takes
 * window element (value & 3) as its winner and lets gradient through iff (value >> 2) & 1;
 * layer 3 = fc1 unit `index` lets gradient through iff value != 0.            */
void oracle_worker_grad(const oracle_dims* d, const double* theta, const double* x, const int32_t* y, int32_t B,
                        const uint8_t* keep, double scale, double* grad, double* loss, uint8_t* code1,
                        double* top1, double* margin1, uint8_t* code2, double* top2, double* margin2,
                        double* hpre_out, double* z_out, const int32_t* forced, int32_t n_forced)
{
    const int H = d->H, W = d->W, C1 = d->C1, C2 = d->C2, F = d->F, NC = d->NC;
    const int H1 = H / 2, W1 = W / 2, H2 = H / 4, W2 = W / 4;
    const int n1 = C1 * H1 * W1, n2 = C2 * H2 * W2;
    const int64_t P = oracle_param_count(d);

    const double* Wc1 = theta;
    const double* bc1 = Wc1 + (int64_t)C1 * 9;
    const double* Wc2 = bc1 + C1;
    const double* bc2 = Wc2 + (int64_t)C2 * C1 * 9;
    const double* Wf1 = bc2 + C2;
    const double* bf1 = Wf1 + (int64_t)F * n2;
    const double* Wf2 = bf1 + F;
    const double* bf2 = Wf2 + (int64_t)NC * F;

    double* gWc1 = grad;
    double* gbc1 = gWc1 + (int64_t)C1 * 9;
    double* gWc2 = gbc1 + C1;
    double* gbc2 = gWc2 + (int64_t)C2 * C1 * 9;
    double* gWf1 = gbc2 + C2;
    double* gbf1 = gWf1 + (int64_t)F * n2;
    double* gWf2 = gbf1 + F;
    double* gbf2 = gWf2 + (int64_t)NC * F;
    memset(grad, 0, sizeof(double) * (size_t)P);

    double* c1 = malloc(sizeof(double) * (size_t)C1 * H * W);
    double* p1 = malloc(sizeof(double) * (size_t)n1);
    double* c2 = malloc(sizeof(double) * (size_t)C2 * H1 * W1);
    double* p2 = malloc(sizeof(double) * (size_t)n2);
    uint8_t* k1 = malloc((size_t)n1);
    uint8_t* k2 = malloc((size_t)n2);
    double* t1 = malloc(sizeof(double) * (size_t)n1);
    double* m1 = malloc(sizeof(double) * (size_t)n1);
    double* t2 = malloc(sizeof(double) * (size_t)n2);
    double* m2 = malloc(sizeof(double) * (size_t)n2);
    double* hpre = malloc(sizeof(double) * (size_t)F);
    double* hd = malloc(sizeof(double) * (size_t)F);
    double* z = malloc(sizeof(double) * (size_t)NC);
    double* dz = malloc(sizeof(double) * (size_t)NC);
    double* dh = malloc(sizeof(double) * (size_t)F);
    double* dp2 = malloc(sizeof(double) * (size_t)n2);
    double* dc2 = malloc(sizeof(double) * (size_t)C2 * H1 * W1);
    double* dp1 = malloc(sizeof(double) * (size_t)n1);
    double* dc1 = malloc(sizeof(double) * (size_t)C1 * H * W);
    uint8_t* g1 = malloc((size_t)n1); /* gradient passes the ReLU under the pool */
    uint8_t* g2 = malloc((size_t)n2);
    uint8_t* g3 = malloc((size_t)F);

    double loss_sum = 0.0;
    for (int s = 0; s < B; ++s) {
        const double* xs = x + (int64_t)s * H * W;
        const uint8_t* ks = keep + (int64_t)s * F;

        /* ---- forward ---- */
        conv3x3(1, C1, H, W, xs, Wc1, bc1, c1);
        relu_pool2(C1, H, W, c1, p1, k1, t1, m1);
        for (int i = 0; i < n1; ++i) g1[i] = t1[i] > 0.0;
        for (int r = 0; r < n_forced; ++r) {
            const int32_t* f = forced + 4 * r;
            if (f[0] != s || f[1] != 1) continue;
            int idx = f[2], o = idx / (H1 * W1), py = (idx / W1) % H1, px = idx % W1, k = f[3] & 3;
            double v = c1[(o * H + 2 * py + k / 2) * W + 2 * px + k % 2];
            k1[idx] = (uint8_t)k;
            g1[idx] = (uint8_t)((f[3] >> 2) & 1);
            p1[idx] = v > 0.0 ? v : 0.0;
        }
        conv3x3(C1, C2, H1, W1, p1, Wc2, bc2, c2);
        relu_pool2(C2, H1, W1, c2, p2, k2, t2, m2);
        for (int i = 0; i < n2; ++i) g2[i] = t2[i] > 0.0;
        for (int r = 0; r < n_forced; ++r) {
            const int32_t* f = forced + 4 * r;
            if (f[0] != s || f[1] != 2) continue;
            int idx = f[2], o = idx / (H2 * W2), py = (idx / W2) % H2, px = idx % W2, k = f[3] & 3;
            double v = c2[(o * H1 + 2 * py + k / 2) * W1 + 2 * px + k % 2];
            k2[idx] = (uint8_t)k;
            g2[idx] = (uint8_t)((f[3] >> 2) & 1);
            p2[idx] = v > 0.0 ? v : 0.0;
        }
        for (int u = 0; u < F; ++u) {
            double acc = bf1[u];
            for (int i = 0; i < n2; ++i) acc += Wf1[(int64_t)u * n2 + i] * p2[i];
            hpre[u] = acc;
            g3[u] = acc > 0.0;
            double r = acc > 0.0 ? acc : 0.0;
            hd[u] = ks[u] ? r * scale : 0.0;
        }
        for (int r = 0; r < n_forced; ++r) {
            const int32_t* f = forced + 4 * r;
            if (f[0] == s && f[1] == 3) g3[f[2]] = f[3] != 0;
        }
        double zmax = -INFINITY;
        for (int j = 0; j < NC; ++j) {
            double acc = bf2[j];
            for (int u = 0; u < F; ++u) acc += Wf2[(int64_t)j * F + u] * hd[u];
            z[j] = acc;
            if (acc > zmax) zmax = acc;
        }
        double se = 0.0;
        for (int j = 0; j < NC; ++j) se += exp(z[j] - zmax);
        double lse = zmax + log(se);
        loss_sum += lse - z[y[s]];

        if (code1) memcpy(code1 + (int64_t)s * n1, k1, (size_t)n1);
        if (top1) memcpy(top1 + (int64_t)s * n1, t1, sizeof(double) * (size_t)n1);
        if (margin1) memcpy(margin1 + (int64_t)s * n1, m1, sizeof(double) * (size_t)n1);
        if (code2) memcpy(code2 + (int64_t)s * n2, k2, (size_t)n2);
        if (top2) memcpy(top2 + (int64_t)s * n2, t2, sizeof(double) * (size_t)n2);
        if (margin2) memcpy(margin2 + (int64_t)s * n2, m2, sizeof(double) * (size_t)n2);
        if (hpre_out) memcpy(hpre_out + (int64_t)s * F, hpre, sizeof(double) * (size_t)F);
        if (z_out) memcpy(z_out + (int64_t)s * NC, z, sizeof(double) * (size_t)NC);

        /* ---- backward: d(mean loss)/d(everything) ---- */
        for (int j = 0; j < NC; ++j) dz[j] = (exp(z[j] - lse) - (j == y[s] ? 1.0 : 0.0)) / (double)B;
        for (int j = 0; j < NC; ++j) {
            gbf2[j] += dz[j];
            for (int u = 0; u < F; ++u) gWf2[(int64_t)j * F + u] += dz[j] * hd[u];
        }
        for (int u = 0; u < F; ++u) {
            double acc = 0.0;
            for (int j = 0; j < NC; ++j) acc += dz[j] * Wf2[(int64_t)j * F + u];
            /* through dropout (same mask and scale), then through ReLU (derivative 0 at 0) */
            dh[u] = (ks[u] && g3[u]) ? acc * scale : 0.0;
        }
        for (int u = 0; u < F; ++u) {
            gbf1[u] += dh[u];
            for (int i = 0; i < n2; ++i) gWf1[(int64_t)u * n2 + i] += dh[u] * p2[i];
        }
        for (int i = 0; i < n2; ++i) {
            double acc = 0.0;
            for (int u = 0; u < F; ++u) acc += dh[u] * Wf1[(int64_t)u * n2 + i];
            dp2[i] = acc;
        }
        /* un-pool + ReLU gate -> gradient w.r.t. conv2 pre-activation */
        memset(dc2, 0, sizeof(double) * (size_t)C2 * H1 * W1);
        for (int o = 0; o < C2; ++o)
            for (int py = 0; py < H2; ++py)
                for (int px = 0; px < W2; ++px) {
                    int idx = (o * H2 + py) * W2 + px;
                    if (g2[idx])
                        dc2[(o * H1 + 2 * py + k2[idx] / 2) * W1 + 2 * px + k2[idx] % 2] = dp2[idx];
                }
        memset(dp1, 0, sizeof(double) * (size_t)n1);
        for (int o = 0; o < C2; ++o)
            for (int yy = 0; yy < H1; ++yy)
                for (int xx = 0; xx < W1; ++xx) {
                    double g = dc2[(o * H1 + yy) * W1 + xx];
                    if (g == 0.0) continue;
                    gbc2[o] += g;
                    for (int c = 0; c < C1; ++c)
                        for (int dy = 0; dy < 3; ++dy)
                            for (int dx = 0; dx < 3; ++dx) {
                                int iy = yy + dy - 1, ix = xx + dx - 1;
                                if (iy < 0 || iy >= H1 || ix < 0 || ix >= W1) continue;
                                int wi = ((o * C1 + c) * 3 + dy) * 3 + dx;
                                gWc2[wi] += g * p1[(c * H1 + iy) * W1 + ix];
                                dp1[(c * H1 + iy) * W1 + ix] += g * Wc2[wi];
                            }
                }
        memset(dc1, 0, sizeof(double) * (size_t)C1 * H * W);
        for (int o = 0; o < C1; ++o)
            for (int py = 0; py < H1; ++py)
                for (int px = 0; px < W1; ++px) {
                    int idx = (o * H1 + py) * W1 + px;
                    if (g1[idx]) dc1[(o * H + 2 * py + k1[idx] / 2) * W + 2 * px + k1[idx] % 2] = dp1[idx];
                }
        for (int o = 0; o < C1; ++o)
            for (int yy = 0; yy < H; ++yy)
                for (int xx = 0; xx < W; ++xx) {
                    double g = dc1[(o * H + yy) * W + xx];
                    if (g == 0.0) continue;
                    gbc1[o] += g;
                    for (int dy = 0; dy < 3; ++dy)
                        for (int dx = 0; dx < 3; ++dx) {
                            int iy = yy + dy - 1, ix = xx + dx - 1;
                            if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                            gWc1[(o * 3 + dy) * 3 + dx] += g * xs[iy * W + ix];
                        }
                }
    }
    *loss = loss_sum / (double)B;

    free(c1); free(p1); free(c2); free(p2); free(k1); free(k2); free(t1); free(m1); free(t2); free(m2);
    free(hpre); free(hd); free(z); free(dz); free(dh); free(dp2); free(dc2); free(dp1); free(dc1); free(g1); free(g2); free(g3);
}

/* n independent workers, each with its own snapshot, minibatch and mask
 * (workers are independent given their snapshot, so the loop may run on
 * several host threads; the arithmetic of each worker is unchanged).
 * theta_of[w] indexes into thetas[.][P]; records are not produced here.
 * Returns the number of host threads used.                               */
int32_t oracle_worker_grads(const oracle_dims* d, int32_t n, const double* thetas, const int32_t* theta_of,
                            const double* x, const int32_t* y, int32_t B, const uint8_t* keep, double scale,
                            double* grads, double* losses, int32_t n_threads)
{
    const int64_t P = oracle_param_count(d);
    const int64_t HW = (int64_t)d->H * d->W;
    int32_t used = 1;
#ifdef _OPENMP
    if (n_threads < 1) n_threads = 1;
    used = n_threads < n ? n_threads : n;
#pragma omp parallel for schedule(dynamic, 1) num_threads(used)
#endif
    for (int32_t w = 0; w < n; ++w)
        oracle_worker_grad(d, thetas + (int64_t)theta_of[w] * P, x + (int64_t)w * B * HW, y + (int64_t)w * B, B,
                           keep + (int64_t)w * B * d->F, scale, grads + (int64_t)w * P, losses + w, NULL, NULL,
                           NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0);
    return used;
}
