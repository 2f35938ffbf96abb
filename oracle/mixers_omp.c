/* fp64 C / OpenMP twin of oracle/mixers.py (test infrastructure only).
 *
 * The numpy oracle stays the parity authority.  This file repeats its definitions as plain loops so that the
 * benchmark can time the same arithmetic on all host cores; tests admit it only while it agrees with the numpy
 * oracle to 1e-12.  Nothing of the HIP library is included, linked or called here, and the library never loads
 * this file: only tests and the cpu_baseline leg of bench.py do (through oracle/omp.py).
 *
 * What each function follows
 *   sa_oracle_delta_steps  Appendix B, "Gated DeltaNet (GDN)" (scalar gate) and "Kimi Delta Attention (KDA)"
 *                          (one gate per key channel): per step  Sbar = decay(S);  u = Sbar^T k;
 *                          S = Sbar + beta k (v - u)^T;  o = scale S^T q  (read-out after the write: the
 *                          reading taken, the paper prints none).
 *   sa_oracle_attn_decode  Appendix B, "Full Attention (FA)" / "Sliding Window Attention (SWA)": softmax attention
 *                          of the newest T tokens over a paged cache, each token seeing the positions
 *                          [max(0, hi - w), hi) with hi = its own position + 1 (w <= 0: all of [0, hi)).
 * bf16 inputs arrive as 16-bit patterns and are widened exactly.  Parallel over (sequence, head) resp.
 * (sequence, KV head); every output element is produced by one thread in a fixed order, so results do not depend on
 * the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen(uint16_t x) {
  uint32_t bits = (uint32_t)x << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

int sa_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* q, k: bf16 [B,T,Hk,dk]; v: bf16 [B,T,H,dv]; alpha: fp32 [B,T,H] or, per_channel, [B,T,H,dk]; beta: fp32 [B,T,H];
 * state: fp32 [B,H,dk,dv]; out: fp64 [B,T,H,dv]; state_out: fp64 [B,H,dk,dv] = the state after n_commit steps.
 * State head h reads q/k head h / (H/Hk).  Returns 0, or -1 on bad sizes / out of memory. */
int sa_oracle_delta_steps(const uint16_t* q, const uint16_t* k, const uint16_t* v, const float* alpha, const float* beta,
                          const float* state, double* out, double* state_out, int B, int T, int H, int Hk, int dk, int dv,
                          double scale, int per_channel, int n_commit) {
  if (B < 0 || T < 1 || H < 1 || Hk < 1 || H % Hk || dk < 1 || dv < 1 || n_commit < 0 || n_commit > T) return -1;
  int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      double* S = (double*)malloc(sizeof(double) * dk * dv);
      double* u = (double*)malloc(sizeof(double) * dv);
      if (!S || !u) {
        failed = 1;
        free(S);
        free(u);
        continue;
      }
      const size_t tile = ((size_t)b * H + h) * dk * dv;
      for (int i = 0; i < dk * dv; ++i) S[i] = (double)state[tile + i];
      if (n_commit == 0)
        for (int i = 0; i < dk * dv; ++i) state_out[tile + i] = S[i];
      const int hk = h / (H / Hk);
      for (int t = 0; t < T; ++t) {
        const size_t bt = (size_t)b * T + t;
        const uint16_t* kt = k + (bt * Hk + hk) * dk;
        const uint16_t* qt = q + (bt * Hk + hk) * dk;
        const uint16_t* vt = v + (bt * H + h) * dv;
        const double bet = (double)beta[bt * H + h];
        /* decay: Sbar = alpha S (scalar) or Sbar[i,:] = alpha_i S[i,:] */
        for (int i = 0; i < dk; ++i) {
          const double a = per_channel ? (double)alpha[(bt * H + h) * dk + i] : (double)alpha[bt * H + h];
          for (int j = 0; j < dv; ++j) S[i * dv + j] *= a;
        }
        /* u = Sbar^T k */
        for (int j = 0; j < dv; ++j) u[j] = 0.0;
        for (int i = 0; i < dk; ++i) {
          const double ki = widen(kt[i]);
          for (int j = 0; j < dv; ++j) u[j] += S[i * dv + j] * ki;
        }
        /* S = Sbar + k (beta (v - u))^T */
        for (int j = 0; j < dv; ++j) u[j] = bet * (widen(vt[j]) - u[j]);
        for (int i = 0; i < dk; ++i) {
          const double ki = widen(kt[i]);
          for (int j = 0; j < dv; ++j) S[i * dv + j] += ki * u[j];
        }
        /* o = scale S^T q, with the state after the write */
        double* o = out + (bt * H + h) * dv;
        for (int j = 0; j < dv; ++j) o[j] = 0.0;
        for (int i = 0; i < dk; ++i) {
          const double qi = widen(qt[i]);
          for (int j = 0; j < dv; ++j) o[j] += S[i * dv + j] * qi;
        }
        for (int j = 0; j < dv; ++j) o[j] *= scale;
        if (t + 1 == n_commit)
          for (int i = 0; i < dk * dv; ++i) state_out[tile + i] = S[i];
      }
      free(S);
      free(u);
    }
  return failed ? -1 : 0;
}

/* q: bf16 [B,T,Hq,D]; kpool, vpool: bf16 [n_pages,Hkv,16*D] blocks whose element (token j, dim d) sits at
 * kmap[j*D+d] resp. vmap[j*D+d] (the caller passes the in-page order: identity maps for logical pools);
 * page_table: int32 [B,max_pages]; seq_lens: int32 [B] (counts the T new tokens); out: fp64 [B,T,Hq,D], rows with
 * no visible position are zeros.  KV head of query head h: h / (Hq/Hkv).  Returns 0; -1 on bad sizes or out of
 * memory; -2 if a visible token sits on an unmapped (negative or too large) page. */
int sa_oracle_attn_decode(const uint16_t* q, const uint16_t* kpool, const uint16_t* vpool, int n_pages, const int32_t* kmap,
                          const int32_t* vmap, const int32_t* page_table, int max_pages, const int32_t* seq_lens, double* out,
                          int B, int T, int Hq, int Hkv, int D, int window, double scale) {
  enum { PAGE = 16 };
  if (B < 0 || T < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || D < 1 || max_pages < 0) return -1;
  const int G = Hq / Hkv;
  int status = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < B; ++b)
    for (int g = 0; g < Hkv; ++g) {
      const int L = seq_lens[b];
      for (int i = 0; i < T; ++i)
        for (int hh = 0; hh < G; ++hh) memset(out + (((size_t)b * T + i) * Hq + g * G + hh) * D, 0, sizeof(double) * D);
      if (L <= 0) continue;
      /* the positions any of the T tokens sees: [lo_all, L) */
      int lo_all = 0;
      if (window > 0) {
        lo_all = L - T + 1 - window;
        if (lo_all < 0) lo_all = 0;
      }
      const int n = L - lo_all;
      double* K = (double*)malloc(sizeof(double) * (size_t)n * D);
      double* V = (double*)malloc(sizeof(double) * (size_t)n * D);
      double* s = (double*)malloc(sizeof(double) * (size_t)n);
      int bad = !K || !V || !s;
      for (int j = lo_all; j < L && !bad; ++j) {
        const int lp = j / PAGE;
        const int phys = lp < max_pages ? page_table[(size_t)b * max_pages + lp] : -1;
        if (phys < 0 || phys >= n_pages) {
          bad = 2;
          break;
        }
        const uint16_t* kb = kpool + ((size_t)phys * Hkv + g) * PAGE * D;
        const uint16_t* vb = vpool + ((size_t)phys * Hkv + g) * PAGE * D;
        for (int d = 0; d < D; ++d) {
          K[(size_t)(j - lo_all) * D + d] = widen(kb[kmap[(j % PAGE) * D + d]]);
          V[(size_t)(j - lo_all) * D + d] = widen(vb[vmap[(j % PAGE) * D + d]]);
        }
      }
      if (bad) {
#pragma omp critical
        status = bad == 2 ? -2 : -1;
      } else {
        for (int i = 0; i < T; ++i) {
          const int hi = L - T + i + 1;
          int lo = 0;
          if (window > 0 && hi - window > 0) lo = hi - window;
          if (hi <= 0 || hi <= lo) continue;
          for (int hh = 0; hh < G; ++hh) {
            const int h = g * G + hh;
            const uint16_t* qr = q + (((size_t)b * T + i) * Hq + h) * D;
            double biggest = -INFINITY;
            for (int j = lo; j < hi; ++j) {
              double acc = 0.0;
              for (int d = 0; d < D; ++d) acc += widen(qr[d]) * K[(size_t)(j - lo_all) * D + d];
              s[j - lo_all] = scale * acc;
              if (s[j - lo_all] > biggest) biggest = s[j - lo_all];
            }
            double total = 0.0;
            for (int j = lo; j < hi; ++j) {
              s[j - lo_all] = exp(s[j - lo_all] - biggest);
              total += s[j - lo_all];
            }
            double* o = out + (((size_t)b * T + i) * Hq + h) * D;
            for (int j = lo; j < hi; ++j) {
              const double w = s[j - lo_all] / total;
              for (int d = 0; d < D; ++d) o[d] += w * V[(size_t)(j - lo_all) * D + d];
            }
          }
        }
      }
      free(K);
      free(V);
      free(s);
    }
  return status;
}
