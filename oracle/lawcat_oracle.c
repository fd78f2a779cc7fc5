/*
 * LAWCAT sequence-mixing oracle: plain, slow, fp64, token by token.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the independent checker for the HIP
 * library; it shares no code with it and must never be called from the product
 * path.  Only the tests, the smoke check and the benchmark's cpu_baseline leg
 * may load it.
 *
 * What it computes (paper section 4):
 *   - section 4.1: causal depthwise Conv1D across tokens, kernel size r+1,
 *       x~_t = sum_{delta=0..r} w_delta * x_{t-delta}   (the "simplest case" sum)
 *     followed by an optional pointwise positive map (1+ELU, named in section 2
 *     as an example of phi).
 *   - section 4.1, optionally: the linear layer with nonlinearity that follows the conv, shared by query and key,
 *       q-dot = phi(q~ Wf), k-dot = phi(k~ Wf)
 *   - section 4.2, KV-state update equation (first equation of 4.2):
 *       S_t = G_t (.) S_{t-1} + k_t^T v_t ,  S_0 = 0 unless a start state is given
 *     with the gate per key channel (G_t = alpha_t^T 1), alpha_t = sigmoid(g_t)^gate_scale,
 *   - section 4.2, normalized output equation (last equation of 4.2):
 *       o_t = q_t S_t / (q_t . z_t + eps) ,  z_t = alpha_t (.) z_{t-1} + k_t
 *     (z_t is the paper's "k^T times 1_{1 x dv}, gated, then mean over dv": with a
 *     per-channel gate all dv columns are identical, so the mean is that column).
 *
 * Every function below is the definition written out: no blocking, no fusion.
 * Pinned by tests/test_oracle_pins.py (brute-force quadratic form, closed forms,
 * invariants); nothing here is "parity unpinned".
 *
 * Build: gcc -O3 -fopenmp -shared -fPIC -o liblawcat_oracle.so lawcat_oracle.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

/* phi: 0 = identity, 1 = 1+ELU (x>0 ? 1+x : exp(x)); section 2, kernel-based linear attention. */
static double feature_map(double x, int kind) {
  if (kind == 1) return x > 0.0 ? 1.0 + x : exp(x);
  return x;
}

/* log(sigmoid(g)), stable on both tails; the gate of section 4.2 is a sigmoid. */
static double log_sigmoid(double g) {
  return g < 0.0 ? g - log1p(exp(g)) : -log1p(exp(-g));
}

/*
 * Section 4.1 direct sum.  x: [B,T,H,d]; w: [H,d,W] with w[..,delta] multiplying x[t-delta];
 * halo: NULL (zeros before the first token) or [B,W-1,H,d], oldest row first, holding
 * the W-1 raw rows that precede x (the "cache limited by the kernel size" of 4.1).
 * y: [B,T,H,d] = phi(conv).
 */
void lawcat_oracle_conv1d_causal(int B, int T, int H, int d, int W, const double* x,
                                 const double* w, const double* halo, int phi, double* y) {
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < T; ++t)
      for (int h = 0; h < H; ++h)
        for (int c = 0; c < d; ++c) {
          double acc = 0.0;
          for (int delta = 0; delta < W; ++delta) {
            int s = t - delta; /* source token */
            double xv;
            if (s >= 0) {
              xv = x[(((size_t)b * T + s) * H + h) * d + c];
            } else if (halo != NULL) {
              int r = (W - 1) + s; /* s = -1 is the newest halo row, index W-2 */
              xv = halo[(((size_t)b * (W - 1) + r) * H + h) * d + c];
            } else {
              xv = 0.0;
            }
            acc += w[((size_t)h * d + c) * W + delta] * xv;
          }
          y[(((size_t)b * T + t) * H + h) * d + c] = feature_map(acc, phi);
        }
}

/*
 * Section 4.1, the layer after the conv: "a linear layer with nonlinearity", the same for the query and the key.
 *   y[b,t,h,f] = phi( sum_c x[b,t,h,c] * wf[h / group, c, f] )
 * x: [B,T,H,d] (the conv output, no nonlinearity applied yet); wf: [H/group, d, d]: one matrix per group of
 * `group` consecutive heads (group = 1 for key heads, Hq/Hkv for query heads, so that a key head and the query
 * heads that read its state share one matrix); y: [B,T,H,d].
 */
void lawcat_oracle_feature_linear(int B, int T, int H, int d, int group, const double* x, const double* wf,
                                  int phi, double* y) {
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < T; ++t)
      for (int h = 0; h < H; ++h) {
        const double* xr = x + (((size_t)b * T + t) * H + h) * d;
        const double* w = wf + (size_t)(h / group) * d * d;
        double* yr = y + (((size_t)b * T + t) * H + h) * d;
        for (int f = 0; f < d; ++f) {
          double acc = 0.0;
          for (int c = 0; c < d; ++c) acc += xr[c] * w[(size_t)c * d + f];
          yr[f] = feature_map(acc, phi);
        }
      }
}

/*
 * Section 4.2, where the gate comes from: "linear layers" followed by the sigmoid; the rank ablation of the
 * appendix says which: two consecutive low-rank linear layers (rank 32 in the distilled models).  The logits
 *   g[b,t,n] = sum_r ( sum_c x[b,t,c] * w1[r,c] ) * w2[n,r]  (+ bias[n])
 * x: [B,T,dm] the layer input; w1: [rank,dm], w2: [N,rank] (out-features x in-features), bias: NULL or [N];
 * N = Hkv * dk, so g is the [B,T,Hkv,dk] gate-logit tensor of the recurrence below.
 */
void lawcat_oracle_gate_project(int B, int T, int dm, int rank, int N, const double* x, const double* w1,
                                const double* w2, const double* bias, double* g) {
#pragma omp parallel for schedule(static)
  for (long long bt = 0; bt < (long long)B * T; ++bt) {
    const double* xr = x + (size_t)bt * dm;
    double* gr = g + (size_t)bt * N;
    double h[1024];
    for (int r = 0; r < rank; ++r) {
      double acc = 0.0;
      for (int c = 0; c < dm; ++c) acc += xr[c] * w1[(size_t)r * dm + c];
      h[r] = acc;
    }
    for (int n = 0; n < N; ++n) {
      double acc = bias ? bias[n] : 0.0;
      for (int r = 0; r < rank; ++r) acc += h[r] * w2[(size_t)n * rank + r];
      gr[n] = acc;
    }
  }
}

/*
 * Section 4.2 recurrence, token by token.
 *   q: [B,T,Hq,dk]  k,g: [B,T,Hkv,dk]  v: [B,T,Hkv,dv]   (q, k are already q-dot, k-dot)
 *   S0: NULL or [B,Hkv,dk,dv];  z0: NULL or [B,Hkv,dk]
 *   o: [B,T,Hq,dv]  den: [B,T,Hq] (q.z + eps)  num: NULL or [B,T,Hq,dv] (q S, before the division)
 *   S_out: [B,Hkv,dk,dv]  z_out: [B,Hkv,dk]
 * Query head h uses the state of kv head h / (Hq/Hkv).
 */
void lawcat_oracle_gla_prefill(int B, int T, int Hq, int Hkv, int dk, int dv, const double* q,
                               const double* k, const double* v, const double* g,
                               double gate_scale, double eps, const double* S0, const double* z0,
                               double* o, double* den, double* num, double* S_out,
                               double* z_out) {
  const int group = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < B; ++b)
    for (int hk = 0; hk < Hkv; ++hk) {
      double* S = (double*)malloc(sizeof(double) * (size_t)dk * dv);
      double* z = (double*)malloc(sizeof(double) * (size_t)dk);
      double* alpha = (double*)malloc(sizeof(double) * (size_t)dk);
      const size_t sidx = ((size_t)b * Hkv + hk);
      for (int c = 0; c < dk; ++c) {
        z[c] = z0 ? z0[sidx * dk + c] : 0.0;
        for (int j = 0; j < dv; ++j) S[(size_t)c * dv + j] = S0 ? S0[(sidx * dk + c) * dv + j] : 0.0;
      }
      for (int t = 0; t < T; ++t) {
        const double* kt = k + (((size_t)b * T + t) * Hkv + hk) * dk;
        const double* gt = g + (((size_t)b * T + t) * Hkv + hk) * dk;
        const double* vt = v + (((size_t)b * T + t) * Hkv + hk) * dv;
        for (int c = 0; c < dk; ++c) alpha[c] = exp(gate_scale * log_sigmoid(gt[c]));
        /* S_t = G_t (.) S_{t-1} + k_t^T v_t ; z_t = alpha_t (.) z_{t-1} + k_t */
        for (int c = 0; c < dk; ++c) {
          double* Sc = S + (size_t)c * dv;
          for (int j = 0; j < dv; ++j) Sc[j] = alpha[c] * Sc[j] + kt[c] * vt[j];
          z[c] = alpha[c] * z[c] + kt[c];
        }
        /* o_t = q_t S_t / (q_t . z_t + eps) for every query head of the group */
        for (int r = 0; r < group; ++r) {
          const int hq = hk * group + r;
          const double* qt = q + (((size_t)b * T + t) * Hq + hq) * dk;
          double* ot = o + (((size_t)b * T + t) * Hq + hq) * dv;
          double dsum = 0.0;
          for (int c = 0; c < dk; ++c) dsum += qt[c] * z[c];
          dsum += eps;
          den[((size_t)b * T + t) * Hq + hq] = dsum;
          for (int j = 0; j < dv; ++j) ot[j] = 0.0;
          for (int c = 0; c < dk; ++c) {
            const double* Sc = S + (size_t)c * dv;
            for (int j = 0; j < dv; ++j) ot[j] += qt[c] * Sc[j];
          }
          if (num) {
            double* nt = num + (((size_t)b * T + t) * Hq + hq) * dv;
            for (int j = 0; j < dv; ++j) nt[j] = ot[j];
          }
          for (int j = 0; j < dv; ++j) ot[j] = ot[j] / dsum;
        }
      }
      for (int c = 0; c < dk; ++c) {
        z_out[sidx * dk + c] = z[c];
        for (int j = 0; j < dv; ++j) S_out[(sidx * dk + c) * dv + j] = S[(size_t)c * dv + j];
      }
      free(S);
      free(z);
      free(alpha);
    }
}

/*
 * Adjoint of lawcat_oracle_gla_prefill (what the layer-wise distillation of section 5 differentiates through):
 * given dO = dL/do, the gradients with respect to q, k, v, the gate logits and the start state.  Token by token:
 * the forward recurrence first, every state kept ([T+1, dk, dv+1] doubles per kv head: small cases only), then
 * backwards with Gr_t = dL/d[S_t | z_t]:
 *   num = q S_t, den = q z_t + eps, o = num / den     =>  dnum = dO / den,  dden = -(dO . o) / den
 *   dq_t  = S_t dnum^T + z_t dden
 *   Gr_t  = alpha_{t+1} (.) Gr_{t+1}  +  sum over the group's query heads of  q_t^T [dnum | dden]
 *   dk_t  = Gr_t [v_t | 1]^T,   dv_t = k_t Gr_t[:, :dv]
 *   dalpha_t[c] = sum_j Gr_t[c, j] [S_{t-1} | z_{t-1}][c, j],   alpha = sigmoid(g)^gate_scale
 *   dg_t  = dalpha_t * gate_scale * alpha_t * (1 - sigmoid(g_t))
 *   dS0, dz0 = alpha_1 (.) Gr_1 (the gradient that reaches the start state)
 * Shapes as in lawcat_oracle_gla_prefill; dS0 [B,Hkv,dk,dv], dz0 [B,Hkv,dk].
 */
void lawcat_oracle_gla_backward(int B, int T, int Hq, int Hkv, int dk, int dv, const double* q, const double* k,
                                const double* v, const double* g, double gate_scale, double eps, const double* S0,
                                const double* z0, const double* dO, double* dq, double* dkk, double* dvv, double* dg,
                                double* dS0, double* dz0) {
  const int group = Hq / Hkv;
  const int w = dv + 1; /* columns of the augmented state [S | z] */
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < B; ++b)
    for (int hk = 0; hk < Hkv; ++hk) {
      const size_t sidx = ((size_t)b * Hkv + hk);
      double* St = (double*)malloc(sizeof(double) * (size_t)(T + 1) * dk * w); /* St[t+1] = state after token t */
      double* al = (double*)malloc(sizeof(double) * (size_t)T * dk);
      double* Gr = (double*)calloc((size_t)dk * w, sizeof(double));
      double* dhat = (double*)malloc(sizeof(double) * (size_t)w);
      for (int c = 0; c < dk; ++c) {
        for (int j = 0; j < dv; ++j) St[(size_t)c * w + j] = S0 ? S0[(sidx * dk + c) * dv + j] : 0.0;
        St[(size_t)c * w + dv] = z0 ? z0[sidx * dk + c] : 0.0;
      }
      for (int t = 0; t < T; ++t) {
        const double* kt = k + (((size_t)b * T + t) * Hkv + hk) * dk;
        const double* gt = g + (((size_t)b * T + t) * Hkv + hk) * dk;
        const double* vt = v + (((size_t)b * T + t) * Hkv + hk) * dv;
        const double* prev = St + (size_t)t * dk * w;
        double* cur = St + (size_t)(t + 1) * dk * w;
        for (int c = 0; c < dk; ++c) {
          const double a = exp(gate_scale * log_sigmoid(gt[c]));
          al[(size_t)t * dk + c] = a;
          for (int j = 0; j < dv; ++j) cur[(size_t)c * w + j] = a * prev[(size_t)c * w + j] + kt[c] * vt[j];
          cur[(size_t)c * w + dv] = a * prev[(size_t)c * w + dv] + kt[c];
        }
      }
      for (int t = T - 1; t >= 0; --t) {
        const double* kt = k + (((size_t)b * T + t) * Hkv + hk) * dk;
        const double* gt = g + (((size_t)b * T + t) * Hkv + hk) * dk;
        const double* vt = v + (((size_t)b * T + t) * Hkv + hk) * dv;
        const double* cur = St + (size_t)(t + 1) * dk * w;
        const double* prev = St + (size_t)t * dk * w;
        /* every query head of the group: its own dq, and its share of Gr_t */
        for (int r = 0; r < group; ++r) {
          const int hq = hk * group + r;
          const double* qt = q + (((size_t)b * T + t) * Hq + hq) * dk;
          const double* dot = dO + (((size_t)b * T + t) * Hq + hq) * dv;
          double* dqt = dq + (((size_t)b * T + t) * Hq + hq) * dk;
          double den = eps;
          for (int c = 0; c < dk; ++c) den += qt[c] * cur[(size_t)c * w + dv];
          double dden = 0.0;
          for (int j = 0; j < dv; ++j) {
            double num = 0.0;
            for (int c = 0; c < dk; ++c) num += qt[c] * cur[(size_t)c * w + j];
            dhat[j] = dot[j] / den;
            dden -= dot[j] * (num / den) / den;
          }
          dhat[dv] = dden;
          for (int c = 0; c < dk; ++c) {
            double acc = 0.0;
            for (int j = 0; j < w; ++j) {
              acc += cur[(size_t)c * w + j] * dhat[j];
              Gr[(size_t)c * w + j] += qt[c] * dhat[j];
            }
            dqt[c] = acc;
          }
        }
        double* dkt = dkk + (((size_t)b * T + t) * Hkv + hk) * dk;
        double* dvt = dvv + (((size_t)b * T + t) * Hkv + hk) * dv;
        double* dgt = dg + (((size_t)b * T + t) * Hkv + hk) * dk;
        for (int j = 0; j < dv; ++j) dvt[j] = 0.0;
        for (int c = 0; c < dk; ++c) {
          double acc = Gr[(size_t)c * w + dv]; /* the column of ones */
          double dal = Gr[(size_t)c * w + dv] * prev[(size_t)c * w + dv];
          for (int j = 0; j < dv; ++j) {
            acc += Gr[(size_t)c * w + j] * vt[j];
            dvt[j] += kt[c] * Gr[(size_t)c * w + j];
            dal += Gr[(size_t)c * w + j] * prev[(size_t)c * w + j];
          }
          dkt[c] = acc;
          const double a = al[(size_t)t * dk + c];
          const double sg = exp(log_sigmoid(gt[c]));
          dgt[c] = dal * gate_scale * a * (1.0 - sg);
          /* what flows on to token t-1 */
          for (int j = 0; j < w; ++j) Gr[(size_t)c * w + j] *= a;
        }
      }
      for (int c = 0; c < dk; ++c) {
        for (int j = 0; j < dv; ++j) dS0[(sidx * dk + c) * dv + j] = Gr[(size_t)c * w + j];
        dz0[sidx * dk + c] = Gr[(size_t)c * w + dv];
      }
      free(St);
      free(al);
      free(Gr);
      free(dhat);
    }
}

/*
 * Adjoint of lawcat_oracle_conv1d_causal: with y = phi(u), u[t,c] = sum_delta w[c,delta] x[t-delta,c] (rows before
 * the first token from the halo), given dy:
 *   du = dy * phi'(u)  (1 for the identity; 1 for u > 0 and exp(u) otherwise for 1 + ELU)
 *   dx[t] = sum_delta w[delta] du[t+delta]   (dhalo likewise for the rows before the first token)
 *   dw[h,c,delta] = sum over batch and tokens of du[t] x[t-delta]
 * dhalo may be NULL (and is ignored when halo is NULL).
 */
void lawcat_oracle_conv1d_backward(int B, int T, int H, int d, int W, const double* x, const double* wt,
                                   const double* halo, int phi, const double* dy, double* dx, double* dw,
                                   double* dhalo) {
  const size_t row = (size_t)H * d;
  for (size_t i = 0; i < (size_t)B * T * row; ++i) dx[i] = 0.0;
  for (size_t i = 0; i < row * W; ++i) dw[i] = 0.0;
  if (dhalo && halo)
    for (size_t i = 0; i < (size_t)B * (W - 1) * row; ++i) dhalo[i] = 0.0;
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < T; ++t)
      for (int h = 0; h < H; ++h)
        for (int c = 0; c < d; ++c) {
          const size_t e = (size_t)h * d + c;
          double u = 0.0;
          for (int dl = 0; dl < W; ++dl) {
            const int s = t - dl;
            double xv = 0.0;
            if (s >= 0) xv = x[((size_t)b * T + s) * row + e];
            else if (halo) xv = halo[((size_t)b * (W - 1) + (W - 1 + s)) * row + e];
            u += wt[e * W + dl] * xv;
          }
          const double du = dy[((size_t)b * T + t) * row + e] * (phi == 1 ? (u > 0.0 ? 1.0 : exp(u)) : 1.0);
          for (int dl = 0; dl < W; ++dl) {
            const int s = t - dl;
            double xv = 0.0;
            if (s >= 0) {
              xv = x[((size_t)b * T + s) * row + e];
              dx[((size_t)b * T + s) * row + e] += wt[e * W + dl] * du;
            } else if (halo) {
              xv = halo[((size_t)b * (W - 1) + (W - 1 + s)) * row + e];
              if (dhalo) dhalo[((size_t)b * (W - 1) + (W - 1 + s)) * row + e] += wt[e * W + dl] * du;
            }
            dw[e * W + dl] += du * xv;
          }
        }
}

int lawcat_oracle_max_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
