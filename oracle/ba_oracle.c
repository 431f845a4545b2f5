/*
 * Block-attention oracle: plain, slow, fp64 CPU definition of the three steps of
 * Block-attention prefill (arXiv 2409.15355).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or import
 * this file; it exists so that tests, the smoke check and the benchmark's
 * cpu_baseline leg have an independent statement of what the method computes.  It
 * shares no code, tables or helpers with the HIP library.
 *
 * Every function is the textbook definition written out, in the order the paper
 * gives the steps (Section 1, "three steps"; Section 2.3, Eq. 1-3; Section 2.5):
 * rotate -> scores -> max -> exp -> weighted sum.  All arithmetic is IEEE double;
 * nothing is rounded in between.  OpenMP only distributes independent output rows.
 *
 * Layouts: every tensor is packed token-major, [tokens][heads][D], D contiguous.
 *
 * Pins (tests/test_oracle_pins.py): one block == causal attention from a library
 * routine; Eq. 2 after Eq. 1 == identity; two-step re-encode == one rotation by the
 * shift; pipeline == dense masked attention built from an explicit T x T mask;
 * first-token rows return v exactly; softmax rows sum to one; and more.  No
 * function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define BAO_LAYOUT_INTERLEAVED 0 /* Eq. 1: pairs (2j, 2j+1)            */
#define BAO_LAYOUT_HALF 1        /* pairs (j, j + D/2), Llama checkpoints */

#define BAO_ROPE_NONE 0  /* q, k arrive already rotated                       */
#define BAO_ROPE_APPLY 1 /* rotate inside (local positions in encode, absolute
                            positions in the final block)                    */

#define BAO_REENC_SHIFT 0    /* cache holds K rotated at old_pos0 + u            */
#define BAO_REENC_ABSOLUTE 1 /* cache holds K with every token at old_pos0       */

int bao_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* theta_j = base^(-2j/D), j = 0 .. D/2-1 (the RoPE frequencies Eq. 1 leaves
 * implicit; the usual definition). */
void bao_theta(double base, int D, double *theta) {
  for (int j = 0; j < D / 2; ++j) theta[j] = pow(base, -2.0 * (double)j / (double)D);
}

static inline void pair_index(int j, int D, int layout, int *a, int *b) {
  if (layout == BAO_LAYOUT_HALF) {
    *a = j;
    *b = j + D / 2;
  } else {
    *a = 2 * j;
    *b = 2 * j + 1;
  }
}

/* Eq. 1 (inverse == 0): y = R(pos) x, each 2x2 block [[c, -s], [s, c]] with angle
 * pos * theta_j.  Eq. 2 (inverse != 0): y = R(pos)^T x, blocks [[c, s], [-s, c]]. */
void bao_rope(const double *x, int D, double pos, const double *theta, int layout, int inverse,
              double *y) {
  for (int j = 0; j < D / 2; ++j) {
    int a, b;
    pair_index(j, D, layout, &a, &b);
    double ang = pos * theta[j];
    double c = cos(ang), s = sin(ang);
    double xa = x[a], xb = x[b];
    if (!inverse) {
      y[a] = c * xa - s * xb;
      y[b] = s * xa + c * xb;
    } else {
      y[a] = c * xa + s * xb;
      y[b] = -s * xa + c * xb;
    }
  }
}

static inline int kv_head_of(int h, int Hq, int Hkv, const int *q_to_kv) {
  return q_to_kv ? q_to_kv[h] : h / (Hq / Hkv);
}

/* softmax(scale * <qhat, K_s>) V over an explicit list of key/value row pointers.
 * Writes o[D]; optionally the max scaled score and the sum of exponentials. */
static void attend_row(const double *qhat, int D, double scale, int n_keys, const double **keys,
                       const double **vals, double *z, double *o, double *m_out, double *l_out) {
  double m = -INFINITY;
  for (int s = 0; s < n_keys; ++s) {
    double dot = 0.0;
    const double *kk = keys[s];
    for (int d = 0; d < D; ++d) dot += qhat[d] * kk[d];
    z[s] = scale * dot;
    if (z[s] > m) m = z[s];
  }
  double l = 0.0;
  for (int d = 0; d < D; ++d) o[d] = 0.0;
  for (int s = 0; s < n_keys; ++s) {
    double p = exp(z[s] - m);
    l += p;
    const double *vv = vals[s];
    for (int d = 0; d < D; ++d) o[d] += p * vv[d];
  }
  for (int d = 0; d < D; ++d) o[d] /= l;
  if (m_out) *m_out = m;
  if (l_out) *l_out = l;
}

/*
 * Step 1 (Section 1, step 1; Section 2.1): every block is encoded on its own.  Token
 * t of block b sees keys s in [c[b], t] only, and positions are local: the first
 * token of a block sits at position 0 (Section 2.3, last paragraph).
 *
 * q [T][Hq][D], k, v [T][Hkv][D]; offs[0..n_blocks] with offs[0] = 0, offs[n_blocks] = T.
 * rows == NULL: all T rows, o is [T][Hq][D].  Otherwise rows[0..n_rows) are token
 * indices and o is [n_rows][Hq][D].
 * k_local (nullable) [T][Hkv][D] receives the rotated keys (the cacheable K).
 * Returns 0, or -1 on bad arguments.
 */
int bao_encode_blocks(const double *q, const double *k, const double *v, int T, int Hq, int Hkv,
                      int D, const int *q_to_kv, double scale, const double *theta, int layout,
                      int n_blocks, const int *offs, int rope_mode, const int *rows, int n_rows,
                      double *o, double *k_local) {
  if (!q || !k || !v || !offs || !o || n_blocks < 0 || offs[0] != 0 || offs[n_blocks] != T) return -1;
  for (int b = 0; b < n_blocks; ++b)
    if (offs[b + 1] < offs[b]) return -1;
  int *block_of = (int *)malloc(sizeof(int) * (size_t)(T > 0 ? T : 1));
  for (int b = 0; b < n_blocks; ++b)
    for (int t = offs[b]; t < offs[b + 1]; ++t) block_of[t] = b;

  /* rotate every key at its local position (or take it as given) */
  double *khat = (double *)malloc(sizeof(double) * (size_t)T * Hkv * D + 8);
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    int pos = t - offs[block_of[t]];
    for (int g = 0; g < Hkv; ++g) {
      const double *src = k + ((size_t)t * Hkv + g) * D;
      double *dst = khat + ((size_t)t * Hkv + g) * D;
      if (rope_mode == BAO_ROPE_APPLY)
        bao_rope(src, D, (double)pos, theta, layout, 0, dst);
      else
        memcpy(dst, src, sizeof(double) * D);
    }
  }
  if (k_local) memcpy(k_local, khat, sizeof(double) * (size_t)T * Hkv * D);

  int n_out = rows ? n_rows : T;
  int bad = 0;
#pragma omp parallel
  {
    double *qhat = (double *)malloc(sizeof(double) * D);
    double *z = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    const double **keys = (const double **)malloc(sizeof(double *) * (size_t)(T > 0 ? T : 1));
    const double **vals = (const double **)malloc(sizeof(double *) * (size_t)(T > 0 ? T : 1));
#pragma omp for schedule(dynamic, 1) collapse(2)
    for (int r = 0; r < n_out; ++r) {
      for (int h = 0; h < Hq; ++h) {
        int t = rows ? rows[r] : r;
        if (t < 0 || t >= T) {
          bad = 1;
          continue;
        }
        int b = block_of[t];
        int start = offs[b];
        int g = kv_head_of(h, Hq, Hkv, q_to_kv);
        const double *qrow = q + ((size_t)t * Hq + h) * D;
        if (rope_mode == BAO_ROPE_APPLY)
          bao_rope(qrow, D, (double)(t - start), theta, layout, 0, qhat);
        else
          memcpy(qhat, qrow, sizeof(double) * D);
        int n = 0;
        for (int s = start; s <= t; ++s, ++n) {
          keys[n] = khat + ((size_t)s * Hkv + g) * D;
          vals[n] = v + ((size_t)s * Hkv + g) * D;
        }
        attend_row(qhat, D, scale, n, keys, vals, z, o + ((size_t)r * Hq + h) * D, NULL, NULL);
      }
    }
    free(qhat);
    free(z);
    free(keys);
    free(vals);
  }
  free(khat);
  free(block_of);
  return bad ? -1 : 0;
}

/*
 * Step 2 (Section 2.3): position re-encoding exactly as the paper states it.  For a
 * cached key of block b at in-block index u:
 *     k0 = R(p_old)^T k          (Eq. 2: set the position back to zero)
 *     k' = R(p_new)   k0         (Eq. 3: rotate to the updated position)
 * SHIFT:    p_old = old_pos0[b] + u,  p_new = new_pos0[b] + u
 * ABSOLUTE: p_old = old_pos0[b],      p_new = new_pos0[b] + u
 * (ABSOLUTE with old_pos0 = 0 is a cache of un-rotated keys.)
 *
 * k_src, k_dst: [n_layers][...tokens...][Hkv][D] with the given layer strides (in
 * elements).  Block b is read from token src_off[b] and written to token dst_off[b].
 * old_pos0 NULL -> 0; new_pos0 NULL -> dst_off.  k_dst may be k_src itself.
 */
int bao_reencode(const double *k_src, double *k_dst, int n_layers, int64_t layer_stride_src,
                 int64_t layer_stride_dst, int Hkv, int D, const double *theta, int layout,
                 int n_blocks, const int *src_off, const int *dst_off, const int *len,
                 const int *old_pos0, const int *new_pos0, int mode) {
  if (!k_src || !k_dst || !src_off || !dst_off || !len) return -1;
#pragma omp parallel
  {
    double *tmp = (double *)malloc(sizeof(double) * D);
    double *out = (double *)malloc(sizeof(double) * D);
#pragma omp for schedule(dynamic, 1) collapse(2)
    for (int layer = 0; layer < n_layers; ++layer) {
      for (int b = 0; b < n_blocks; ++b) {
        double p0_old = old_pos0 ? (double)old_pos0[b] : 0.0;
        double p0_new = new_pos0 ? (double)new_pos0[b] : (double)dst_off[b];
        for (int u = 0; u < len[b]; ++u) {
          double p_old = (mode == BAO_REENC_SHIFT) ? p0_old + u : p0_old;
          double p_new = p0_new + u;
          for (int g = 0; g < Hkv; ++g) {
            const double *src =
                k_src + (size_t)layer * layer_stride_src + ((size_t)(src_off[b] + u) * Hkv + g) * D;
            double *dst =
                k_dst + (size_t)layer * layer_stride_dst + ((size_t)(dst_off[b] + u) * Hkv + g) * D;
            bao_rope(src, D, p_old, theta, layout, 1, tmp); /* Eq. 2 */
            bao_rope(tmp, D, p_new, theta, layout, 0, out); /* Eq. 3 */
            memcpy(dst, out, sizeof(double) * D);
          }
        }
      }
    }
    free(tmp);
    free(out);
  }
  return 0;
}

/*
 * Step 3 (Section 1, step 3; Section 2.5): the final block attends to every cached,
 * re-encoded context key and causally to itself.
 *
 * Prompt n owns final-block rows [cu_q[n], cu_q[n+1]) of q_f/k_f/v_f and context rows
 * [cu_ctx[n], cu_ctx[n+1]) of k_ctx/v_ctx.  Final-block token i sits at absolute
 * position pos0 + i with pos0 = q_pos0[n], or the prompt's context length if q_pos0
 * is NULL.  Context keys are used as given.  With BAO_ROPE_APPLY, q_f and k_f are
 * rotated at their absolute positions first.
 * rows == NULL: all cu_q[n_prompts] rows; else packed final-block row indices.
 * m_out / l_out (nullable) [n_out][Hq]: max scaled score and sum of exponentials.
 */
int bao_final_block(const double *q_f, const double *k_ctx, const double *v_ctx, const double *k_f,
                    const double *v_f, int Hq, int Hkv, int D, const int *q_to_kv, double scale,
                    const double *theta, int layout, int n_prompts, const int *cu_q,
                    const int *cu_ctx, const int *q_pos0, int rope_mode, const int *rows,
                    int n_rows, double *o, double *m_out, double *l_out) {
  if (!q_f || !k_f || !v_f || !cu_q || !cu_ctx || !o || n_prompts < 0) return -1;
  int Lq_total = cu_q[n_prompts];
  int max_keys = 1;
  int *prompt_of = (int *)malloc(sizeof(int) * (size_t)(Lq_total > 0 ? Lq_total : 1));
  for (int n = 0; n < n_prompts; ++n) {
    if (cu_q[n + 1] < cu_q[n] || cu_ctx[n + 1] < cu_ctx[n]) {
      free(prompt_of);
      return -1;
    }
    for (int i = cu_q[n]; i < cu_q[n + 1]; ++i) prompt_of[i] = n;
    int keys = (cu_ctx[n + 1] - cu_ctx[n]) + (cu_q[n + 1] - cu_q[n]);
    if (keys > max_keys) max_keys = keys;
  }
  /* rotate the final block's own keys at their absolute positions */
  double *kfhat = (double *)malloc(sizeof(double) * (size_t)Lq_total * Hkv * D + 8);
#pragma omp parallel for schedule(static)
  for (int i = 0; i < Lq_total; ++i) {
    int n = prompt_of[i];
    int pos0 = q_pos0 ? q_pos0[n] : cu_ctx[n + 1] - cu_ctx[n];
    int pos = pos0 + (i - cu_q[n]);
    for (int g = 0; g < Hkv; ++g) {
      const double *src = k_f + ((size_t)i * Hkv + g) * D;
      double *dst = kfhat + ((size_t)i * Hkv + g) * D;
      if (rope_mode == BAO_ROPE_APPLY)
        bao_rope(src, D, (double)pos, theta, layout, 0, dst);
      else
        memcpy(dst, src, sizeof(double) * D);
    }
  }
  int n_out = rows ? n_rows : Lq_total;
  int bad = 0;
#pragma omp parallel
  {
    double *qhat = (double *)malloc(sizeof(double) * D);
    double *z = (double *)malloc(sizeof(double) * (size_t)max_keys);
    const double **keys = (const double **)malloc(sizeof(double *) * (size_t)max_keys);
    const double **vals = (const double **)malloc(sizeof(double *) * (size_t)max_keys);
#pragma omp for schedule(dynamic, 1) collapse(2)
    for (int r = 0; r < n_out; ++r) {
      for (int h = 0; h < Hq; ++h) {
        int i = rows ? rows[r] : r;
        if (i < 0 || i >= Lq_total) {
          bad = 1;
          continue;
        }
        int n = prompt_of[i];
        int g = kv_head_of(h, Hq, Hkv, q_to_kv);
        int pos0 = q_pos0 ? q_pos0[n] : cu_ctx[n + 1] - cu_ctx[n];
        const double *qrow = q_f + ((size_t)i * Hq + h) * D;
        if (rope_mode == BAO_ROPE_APPLY)
          bao_rope(qrow, D, (double)(pos0 + i - cu_q[n]), theta, layout, 0, qhat);
        else
          memcpy(qhat, qrow, sizeof(double) * D);
        int cnt = 0;
        for (int s = cu_ctx[n]; s < cu_ctx[n + 1]; ++s, ++cnt) { /* all context keys */
          keys[cnt] = k_ctx + ((size_t)s * Hkv + g) * D;
          vals[cnt] = v_ctx + ((size_t)s * Hkv + g) * D;
        }
        for (int s = cu_q[n]; s <= i; ++s, ++cnt) { /* own block, causal */
          keys[cnt] = kfhat + ((size_t)s * Hkv + g) * D;
          vals[cnt] = v_f + ((size_t)s * Hkv + g) * D;
        }
        attend_row(qhat, D, scale, cnt, keys, vals, z, o + ((size_t)r * Hq + h) * D,
                   m_out ? m_out + (size_t)r * Hq + h : NULL,
                   l_out ? l_out + (size_t)r * Hq + h : NULL);
      }
    }
    free(qhat);
    free(z);
    free(keys);
    free(vals);
  }
  free(kfhat);
  free(prompt_of);
  return bad ? -1 : 0;
}
