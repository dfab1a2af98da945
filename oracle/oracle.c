/*
 * CPU oracle for the parallel-verification step of collaborative speculative
 * inference.  TEST INFRASTRUCTURE ONLY: it exists to define what the GPU library
 * must compute and is called from tests/, the smoke check and the benchmark's
 * cpu_baseline leg.  It shares no code with the HIP path and is never used to
 * produce a product result.
 *
 * Everything is the plain definition, in fp64, on inputs upcast exactly
 * (bf16 -> fp64 is exact).  No tiling, no online rescaling, no fusion.  OpenMP is
 * used only across independent units (request x head, request).
 *
 *   oracle_verify_attn  - masked softmax attention of the draft queries over the
 *                         cached context plus their draft ancestors (Section 2.1:
 *                         the target model scores all draft tokens in one parallel
 *                         pass; draft sequences merged into a tree keep causal
 *                         dependencies through a tree-attention mask).
 *   oracle_fuse_drafts  - confidence-based token fusion (Algorithm 1, TokenFusion;
 *                         Eq. 4 first line): keep the token whose drafter reported
 *                         the highest probability.
 *   oracle_accept       - acceptance-rejection of Section 2.1: accept x_i when
 *                         q_i(x_i) <= o_i(x_i), otherwise reject with probability
 *                         1 - o_i(x_i)/q_i(x_i); the first rejection discards the
 *                         rest and a replacement is drawn from
 *                         norm(max(0, o_i - q_i)); if nothing is rejected one more
 *                         token is drawn from the target distribution.
 *   oracle_accept_greedy - the same walk under greedy sampling, the decoding rule of
 *                         the paper's experiments (Section 6.1, experiment settings):
 *                         a draft token is kept when it is the target's most likely
 *                         token at its position; the first mismatch is replaced by
 *                         that most likely token.
 *   oracle_adaptive_speculation - the draft-length adjustment that precedes
 *                         verification (Algorithm 2, AdaptiveSpeculation): while the
 *                         batch's draft tokens exceed the verification budget, the
 *                         request with the most draft tokens gives one up.
 *   oracle_compact_kv    - after a draft tree has been verified, the K/V entries of the
 *                         accepted path are moved to consecutive cache positions so
 *                         that the next step sees an ordinary linear context (the paper
 *                         only says verified drafts return to the request pool,
 *                         Section 4.1; the data movement is this build's reading).
 *   oracle_lm_head      - the projection that produces the logits the acceptance step reads
 *                         (Section 3.1: verification on the target model is dominated by
 *                         matrix-matrix products): logits = hidden x weight^T, rounded to
 *                         bf16, with each row's softmax statistics (maximum and
 *                         sum of exp((l - max)/T) over the rounded logits).
 *   oracle_routing_scores - the routing-score update that follows acceptance
 *                         (Section 4.1, Eq. 1 and Eq. 2): per drafter, the mean over
 *                         draft positions of the normalised harmonic combination of
 *                         its confidence and the cosine similarity between its token's
 *                         embedding and the accepted token's embedding.
 *
 * Pins: tests/test_oracle_*.py (closed forms, chi-square, brute force on tiny
 * vocabularies, library SDPA on the causal special case, tree/path equivalence).
 * Parts with no pin are listed as "parity unpinned" in the test files; at the
 * time of writing every exported function has at least one pin.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_BF16 0
#define ORACLE_F32 1

static inline double bf16_to_double(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

static inline double load_logit(const void* base, int dtype, int64_t idx) {
  if (dtype == ORACLE_BF16) return bf16_to_double(((const uint16_t*)base)[idx]);
  return (double)((const float*)base)[idx];
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* ------------------------------------------------------------------------- */
/* attention                                                                  */
/* ------------------------------------------------------------------------- */
/*
 * q            [total_q, Hq, D] bf16 bits, request b owns rows q_offsets[b]..q_offsets[b+1)
 * k_pool/v_pool[num_pages, Hkv, page_size, D] bf16 bits
 * block_table  [B, max_pages] logical page -> pool page
 * ctx_len      [B] committed tokens; draft node j's K/V sit at logical position ctx_len[b]+j
 * parent       [total_q] parent node inside the request (-1 = child of the committed
 *              prefix), or NULL for a linear draft (node j's parent is j-1)
 * out          [total_q, Hq, D] fp64; lse [total_q, Hq] fp64 or NULL
 *
 * Query node i of request b attends to every committed position and to the draft
 * positions of i itself and of its ancestors.
 */
int oracle_verify_attn(int B, int Hq, int Hkv, int D, int page_size, int max_pages,
                       const uint16_t* q, const uint16_t* k_pool, const uint16_t* v_pool,
                       const int32_t* block_table, const int32_t* ctx_len,
                       const int32_t* q_offsets, const int32_t* parent, double scale,
                       double* out, double* lse) {
  if (Hkv <= 0 || Hq % Hkv != 0) return -2;
  const int G = Hq / Hkv;
  int status = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    for (int h = 0; h < Hq; ++h) {
      const int n = q_offsets[b + 1] - q_offsets[b];
      const int ctx = ctx_len[b];
      const int L = ctx + n;
      const int kvh = h / G;
      double* s = (double*)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
      char* allowed = (char*)malloc((size_t)(n > 0 ? n : 1));
      if (!s || !allowed) { status = -7; free(s); free(allowed); continue; }
      for (int i = 0; i < n; ++i) {
        /* ancestor-or-self set of node i among the draft positions */
        memset(allowed, 0, (size_t)n);
        if (parent) {
          int a = i, guard = 0;
          while (a >= 0 && guard++ <= n) { allowed[a] = 1; a = parent[q_offsets[b] + a]; }
        } else {
          for (int j = 0; j <= i; ++j) allowed[j] = 1;
        }
        const uint16_t* qv = q + ((int64_t)(q_offsets[b] + i) * Hq + h) * D;
        double m = -INFINITY;
        for (int t = 0; t < L; ++t) {
          if (t >= ctx && !allowed[t - ctx]) { s[t] = -INFINITY; continue; }
          const int64_t pg = block_table[(int64_t)b * max_pages + t / page_size];
          const uint16_t* kv = k_pool + ((pg * Hkv + kvh) * page_size + t % page_size) * D;
          double dot = 0.0;
          for (int d = 0; d < D; ++d) dot += bf16_to_double(qv[d]) * bf16_to_double(kv[d]);
          s[t] = scale * dot;
          if (s[t] > m) m = s[t];
        }
        double denom = 0.0;
        for (int t = 0; t < L; ++t) {
          s[t] = (s[t] == -INFINITY) ? 0.0 : exp(s[t] - m);
          denom += s[t];
        }
        double* o = out + ((int64_t)(q_offsets[b] + i) * Hq + h) * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int t = 0; t < L; ++t) {
          if (s[t] == 0.0) continue;
          const int64_t pg = block_table[(int64_t)b * max_pages + t / page_size];
          const uint16_t* vv = v_pool + ((pg * Hkv + kvh) * page_size + t % page_size) * D;
          for (int d = 0; d < D; ++d) o[d] += s[t] * bf16_to_double(vv[d]);
        }
        for (int d = 0; d < D; ++d) o[d] /= denom;
        if (lse) lse[(int64_t)(q_offsets[b] + i) * Hq + h] = m + log(denom);
      }
      free(s);
      free(allowed);
    }
  }
  return status;
}

/* ------------------------------------------------------------------------- */
/* softmax of one row of logits at temperature T, in fp64                      */
/* ------------------------------------------------------------------------- */
static void softmax_row(const void* logits, int dtype, int64_t row, int V, double T, double* prob) {
  double m = -INFINITY;
  for (int v = 0; v < V; ++v) {
    prob[v] = load_logit(logits, dtype, row * V + v) / T;
    if (prob[v] > m) m = prob[v];
  }
  double Z = 0.0;
  for (int v = 0; v < V; ++v) { prob[v] = exp(prob[v] - m); Z += prob[v]; }
  for (int v = 0; v < V; ++v) prob[v] /= Z;
}

/* ------------------------------------------------------------------------- */
/* fusion                                                                     */
/* ------------------------------------------------------------------------- */
/*
 * mode 0 (ARGMAX, the paper's rule): winner = the drafter with the largest reported
 * confidence at that position (first one on ties); fused token = that drafter's
 * token; q_row = row of that drafter's logits in draft_logits.
 * mode 1 (MIXTURE, the "weighted averaging of distributions" ensemble of Section
 * 2.2): fused_probs = sum_n w_n softmax(logits_n / T), w_n = conf_n / sum conf
 * (uniform weights when every confidence is zero); winner/fused_token as ARGMAX;
 * q_row = b*k_max + i (row of fused_probs).
 * Positions i >= k_len[b] are written as -1 and their fused_probs rows as zeros.
 */
int oracle_fuse_drafts(int B, int k_max, int N, int V, const int32_t* k_len, const float* conf,
                       const int32_t* draft_tokens, const void* draft_logits, int ldt,
                       double temperature, int mode, int32_t* fused_token, int32_t* winner,
                       int32_t* q_row, double* fused_probs) {
  if (N <= 0) return -2;
  if (mode == 1 && (!draft_logits || !fused_probs)) return -1;
  double* tmp = (mode == 1) ? (double*)malloc(sizeof(double) * (size_t)V) : NULL;
  for (int b = 0; b < B; ++b) {
    for (int i = 0; i < k_max; ++i) {
      const int64_t pos = (int64_t)b * k_max + i;
      if (i >= k_len[b]) {
        fused_token[pos] = -1; winner[pos] = -1; q_row[pos] = -1;
        if (mode == 1) for (int v = 0; v < V; ++v) fused_probs[pos * V + v] = 0.0;
        continue;
      }
      int best = 0;
      for (int n = 1; n < N; ++n)
        if (conf[pos * N + n] > conf[pos * N + best]) best = n;
      winner[pos] = best;
      fused_token[pos] = draft_tokens[pos * N + best];
      if (mode == 0) {
        q_row[pos] = (int32_t)(pos * N + best);
      } else {
        q_row[pos] = (int32_t)pos;
        double csum = 0.0;
        for (int n = 0; n < N; ++n) csum += (double)conf[pos * N + n];
        for (int v = 0; v < V; ++v) fused_probs[pos * V + v] = 0.0;
        for (int n = 0; n < N; ++n) {
          const double w = (csum > 0.0) ? (double)conf[pos * N + n] / csum : 1.0 / N;
          softmax_row(draft_logits, ldt, pos * N + n, V, temperature, tmp);
          for (int v = 0; v < V; ++v) fused_probs[pos * V + v] += w * tmp[v];
        }
      }
    }
  }
  free(tmp);
  return 0;
}

/* ------------------------------------------------------------------------- */
/* acceptance                                                                 */
/* ------------------------------------------------------------------------- */
/* Smallest index t whose inclusive prefix sum exceeds u * (sum of w); when rounding
 * leaves none, the last index with positive weight.  *tie is set when u lies within
 * eps of the normalised prefix on either side of t. */
static int inv_cdf(const double* w, int V, double u, double eps, int* tie) {
  double W = 0.0;
  for (int v = 0; v < V; ++v) W += w[v];
  const double target = u * W;
  double acc = 0.0, before = 0.0;
  int t = -1, last_pos = -1;
  for (int v = 0; v < V; ++v) {
    if (w[v] > 0.0) last_pos = v;
    before = acc;
    acc += w[v];
    if (acc > target) { t = v; break; }
  }
  if (t < 0) { t = last_pos < 0 ? V - 1 : last_pos; *tie = 1; return t; }
  if (fabs(acc / W - u) < eps || (before > 0.0 && fabs(before / W - u) < eps)) *tie = 1;
  return t;
}

/*
 * node_offsets [B+1]; parent [total] or NULL (linear chain); draft_tokens [total];
 * target_logits [total + B, V]: request b owns rows node_offsets[b]+b ..., local row 0
 *   is the target distribution after the committed prefix, local row 1+j after node j;
 * draft_q [n_q_rows, V]: logits (qkind 0) or probabilities (qkind 1);
 * q_row [total]: row of draft_q that node j's token was drawn from (siblings share it);
 * u_accept [total], u_resample [B] in [0,1).
 *
 * Walk (reduces to the linear rule of Section 2.1 when every node has one child;
 * the extension to several i.i.d. sibling drafts is the recursive rejection used
 * for draft trees, a reading the paper leaves open): cur = committed prefix, r =
 * target distribution after cur.  For each child c of cur in index order: accept
 * when u_accept[c] < r(x_c)/q(x_c) and descend (r = target distribution after c);
 * otherwise r <- norm(max(0, r - q)).  When cur has no child, or all were rejected,
 * emit inv_cdf(r, u_resample[b]).
 *
 * Outputs: accept_len [B] (number of accepted drafts), out_tokens [B, out_stride]
 * (accepted draft tokens then the emitted one), stop_node [B] (last accepted node
 * or -1), dbg_ratio [total] (ratio compared at each visited node, NaN elsewhere),
 * near_tie [B] (1 when any decision of the request lay within tie_eps of flipping).
 */
int oracle_accept(int B, int V, const int32_t* node_offsets, const int32_t* parent,
                  const int32_t* draft_tokens, const void* target_logits, int tdt,
                  const void* draft_q, int qdt, int qkind, const int32_t* q_row,
                  double temperature, const float* u_accept, const float* u_resample,
                  int32_t* accept_len, int32_t* out_tokens, int out_stride, int32_t* stop_node,
                  double* dbg_ratio, int32_t* near_tie, double tie_eps) {
  int status = 0;
  if (dbg_ratio) {
    const int total = node_offsets[B];
    for (int i = 0; i < total; ++i) dbg_ratio[i] = NAN;
  }
#pragma omp parallel for schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    const int o = node_offsets[b];
    const int n = node_offsets[b + 1] - o;
    const int64_t trow0 = (int64_t)o + b;
    double* r = (double*)malloc(sizeof(double) * (size_t)V);
    double* qv = (double*)malloc(sizeof(double) * (size_t)V);
    if (!r || !qv) { status = -7; free(r); free(qv); continue; }
    int cur = -1, depth = 0, tie = 0;
    softmax_row(target_logits, tdt, trow0, V, temperature, r);
    for (;;) {
      int accepted_child = -1, have_q = 0, n_children = 0;
      for (int c = cur + 1; c < n; ++c) { /* parent[c] < c, so children follow cur */
        const int pc = parent ? parent[o + c] : c - 1;
        if (pc != cur) continue;
        ++n_children;
        if (!have_q) {
          const int64_t qr = q_row[o + c];
          if (qkind == 0) softmax_row(draft_q, qdt, qr, V, temperature, qv);
          else for (int v = 0; v < V; ++v) qv[v] = load_logit(draft_q, qdt, qr * V + v);
          have_q = 1;
        }
        const int x = draft_tokens[o + c];
        const double rx = r[x], qx = qv[x];
        double ratio;
        if (qx > 0.0) ratio = rx / qx;
        else ratio = (rx > 0.0) ? INFINITY : 0.0;
        if (dbg_ratio) dbg_ratio[o + c] = ratio;
        const double u = (double)u_accept[o + c];
        if (fabs(ratio - u) < tie_eps) tie = 1;
        if (u < ratio) { accepted_child = c; break; }
        /* rejected: residual distribution */
        double R = 0.0;
        for (int v = 0; v < V; ++v) { const double d = r[v] - qv[v]; R += (d > 0.0) ? d : 0.0; }
        if (R > 0.0)
          for (int v = 0; v < V; ++v) { const double d = r[v] - qv[v]; r[v] = (d > 0.0) ? d / R : 0.0; }
      }
      if (accepted_child >= 0) {
        if (depth < out_stride) out_tokens[(int64_t)b * out_stride + depth] = draft_tokens[o + accepted_child];
        ++depth;
        cur = accepted_child;
        softmax_row(target_logits, tdt, trow0 + 1 + cur, V, temperature, r);
        continue;
      }
      (void)n_children;
      const int t = inv_cdf(r, V, (double)u_resample[b], tie_eps, &tie);
      if (depth < out_stride) out_tokens[(int64_t)b * out_stride + depth] = t;
      break;
    }
    accept_len[b] = depth;
    if (stop_node) stop_node[b] = cur;
    if (near_tie) near_tie[b] = tie;
    free(r);
    free(qv);
  }
  return status;
}

/* ------------------------------------------------------------------------- */
/* greedy verification                                                         */
/* ------------------------------------------------------------------------- */
/* Index of the largest logit of a row; the lowest index wins among equal values.
 * A value replaces the running best only when strictly greater, so NaN entries
 * never win and a row without any finite entry gives index 0. */
static int argmax_row(const void* logits, int dtype, int64_t row, int V) {
  double best = -INFINITY;
  int idx = 0;
  for (int v = 0; v < V; ++v) {
    const double x = load_logit(logits, dtype, row * (int64_t)V + v);
    if (x > best) { best = x; idx = v; }
  }
  return idx;
}

/*
 * Greedy verification (Section 6.1: draft generation and verification both use
 * greedy sampling).  Same inputs as oracle_accept without draft distributions or
 * uniforms.  cur = committed prefix; g = argmax of the target row after cur.  The
 * first child c of cur (index order) with draft_tokens[c] == g is accepted and the
 * walk descends; when cur has no such child, g is emitted and the walk stops.
 * row_argmax [total + B] (optional) receives the argmax of every target row.
 */
int oracle_accept_greedy(int B, int V, const int32_t* node_offsets, const int32_t* parent,
                         const int32_t* draft_tokens, const void* target_logits, int tdt,
                         int32_t* accept_len, int32_t* out_tokens, int out_stride,
                         int32_t* stop_node, int32_t* row_argmax) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    const int o = node_offsets[b];
    const int n = node_offsets[b + 1] - o;
    const int64_t trow0 = (int64_t)o + b;
    if (row_argmax)
      for (int i = 0; i <= n; ++i) row_argmax[trow0 + i] = argmax_row(target_logits, tdt, trow0 + i, V);
    int cur = -1, depth = 0;
    for (;;) {
      const int g = argmax_row(target_logits, tdt, trow0 + 1 + cur, V);
      int accepted_child = -1;
      for (int c = cur + 1; c < n; ++c) {
        const int pc = parent ? parent[o + c] : c - 1;
        if (pc == cur && draft_tokens[o + c] == g) { accepted_child = c; break; }
      }
      if (accepted_child < 0) {
        if (depth < out_stride) out_tokens[(int64_t)b * out_stride + depth] = g;
        break;
      }
      if (depth < out_stride) out_tokens[(int64_t)b * out_stride + depth] = g;
      ++depth;
      cur = accepted_child;
    }
    accept_len[b] = depth;
    if (stop_node) stop_node[b] = cur;
  }
  return 0;
}

/* ------------------------------------------------------------------------- */
/* routing scores                                                              */
/* ------------------------------------------------------------------------- */
/*
 * Eq. 1: d[b,i,n] = cos(H(accepted token i of request b), H(draft_tokens[b,i,n])) for
 * positions i < accept_len[b] (0-based: the positions whose draft was accepted), 0
 * otherwise.  Eq. 2: scores[b,n] = (1/K) sum_i c d / (c d + (1-c)(1-d)), K = k_len[b].
 * Readings where the paper is silent: a negative cosine counts as 0 (Eq. 2 takes values in
 * (0,1)); a zero embedding row gives cosine 0; a term whose denominator is not positive
 * (c = 1, d = 0 or c = 0, d = 1) is 0; K = 0 gives score 0.
 * conf, draft_tokens: [B, k_max, N]; out_tokens: [B, out_stride]; embedding: [V, E].
 */
int oracle_routing_scores(int B, int k_max, int N, int V, int E, const int32_t* k_len, const float* conf,
                          const int32_t* draft_tokens, const int32_t* accept_len, const int32_t* out_tokens,
                          int out_stride, const void* embedding, int edt, double* scores) {
  (void)V;
#pragma omp parallel for schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    const int K = k_len[b];
    for (int n = 0; n < N; ++n) {
      double sum = 0.0;
      for (int i = 0; i < K && i < k_max; ++i) {
        double d = 0.0;
        if (i < accept_len[b]) {
          const int64_t ra = (int64_t)out_tokens[(int64_t)b * out_stride + i] * E;
          const int64_t rx = (int64_t)draft_tokens[((int64_t)b * k_max + i) * N + n] * E;
          double dot = 0.0, na = 0.0, nx = 0.0;
          for (int e = 0; e < E; ++e) {
            const double a = load_logit(embedding, edt, ra + e), x = load_logit(embedding, edt, rx + e);
            dot += a * x; na += a * a; nx += x * x;
          }
          if (na > 0.0 && nx > 0.0) d = dot / (sqrt(na) * sqrt(nx));
          if (d < 0.0) d = 0.0;
          if (d > 1.0) d = 1.0;                 /* rounding of identical rows */
        }
        const double c = (double)conf[((int64_t)b * k_max + i) * N + n];
        const double den = c * d + (1.0 - c) * (1.0 - d);
        if (den > 0.0) sum += c * d / den;
      }
      scores[(int64_t)b * N + n] = (K > 0) ? sum / (double)K : 0.0;
    }
  }
  return 0;
}

/* ------------------------------------------------------------------------- */
/* adaptive speculation                                                        */
/* ------------------------------------------------------------------------- */
/*
 * Algorithm 2, AdaptiveSpeculation(B, Gamma_max): while sum_i b_i gamma_i > Gamma_max, take
 * j = argmax_i gamma_i over the requests of the batch (b_i = 1) and decrement gamma_j.
 * Readings where the paper is silent: ties go to the lowest index; a request keeps at least one
 * draft token (the constraint gamma_i >= 1 of the batch formulation, Section 4.3), so the loop
 * also stops when every request of the batch is at 1; requests outside the batch are untouched.
 * in_batch may be NULL (all requests are in the batch).  Returns the final sum over the batch.
 */
long long oracle_adaptive_speculation(int R, const int32_t* gamma_in, const int32_t* in_batch,
                                      long long gamma_max_total, int32_t* gamma_out) {
  long long sum = 0;
  for (int i = 0; i < R; ++i) {
    gamma_out[i] = gamma_in[i];
    if (!in_batch || in_batch[i]) sum += gamma_in[i];
  }
  while (sum > gamma_max_total) {
    int j = -1;
    for (int i = 0; i < R; ++i) {
      if (in_batch && !in_batch[i]) continue;
      if (j < 0 || gamma_out[i] > gamma_out[j]) j = i;
    }
    if (j < 0 || gamma_out[j] <= 1) break;
    gamma_out[j] -= 1;
    sum -= 1;
  }
  return sum;
}

/* ------------------------------------------------------------------------- */
/* accepted-path compaction of the paged KV cache                              */
/* ------------------------------------------------------------------------- */
/*
 * Request b holds its n[b] draft nodes at logical positions ctx_len[b] + j of its paged cache.
 * With stop_node[b] the last accepted node (-1: none) the accepted path is the chain of ancestors
 * root .. stop_node; its d-th node (d = 0 ..) moves from position ctx + node to position ctx + d,
 * for both pools and every KV head.  All sources are read before anything is written.
 * Pools: [num_pages, Hkv, page, D] 16-bit elements; block_table [B, max_pages].
 * Returns the depth of the path in new_len[b] = ctx_len[b] + depth (optional).
 */
int oracle_compact_kv(int B, int Hkv, int D, int page, int max_pages, uint16_t* k_pool, uint16_t* v_pool,
                      const int32_t* block_table, const int32_t* ctx_len, const int32_t* q_offsets,
                      const int32_t* parent, const int32_t* stop_node, int32_t* new_len) {
  for (int b = 0; b < B; ++b) {
    const int o = q_offsets[b], n = q_offsets[b + 1] - o;
    int* path = (int*)malloc(sizeof(int) * (size_t)(n > 0 ? n : 1));   /* a path has at most n nodes */
    if (!path) return -7;
    int depth = 0;
    for (int a = stop_node[b]; a >= 0 && a < n && depth < n; a = parent ? parent[o + a] : a - 1) path[depth++] = a;
    /* path[] runs leaf -> root; position d from the root is path[depth - 1 - d] */
    const size_t row = (size_t)D;
    uint16_t* tmp = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)(depth > 0 ? depth : 1) * 2 * Hkv * row);
    if (!tmp) { free(path); return -7; }
    for (int d = 0; d < depth; ++d) {
      const int pos = ctx_len[b] + path[depth - 1 - d];
      const int64_t pg = block_table[(int64_t)b * max_pages + pos / page];
      for (int h = 0; h < Hkv; ++h) {
        const int64_t src = ((pg * Hkv + h) * page + pos % page) * (int64_t)D;
        memcpy(tmp + ((size_t)(d * 2 + 0) * Hkv + h) * row, k_pool + src, sizeof(uint16_t) * row);
        memcpy(tmp + ((size_t)(d * 2 + 1) * Hkv + h) * row, v_pool + src, sizeof(uint16_t) * row);
      }
    }
    for (int d = 0; d < depth; ++d) {
      const int pos = ctx_len[b] + d;
      const int64_t pg = block_table[(int64_t)b * max_pages + pos / page];
      for (int h = 0; h < Hkv; ++h) {
        const int64_t dst = ((pg * Hkv + h) * page + pos % page) * (int64_t)D;
        memcpy(k_pool + dst, tmp + ((size_t)(d * 2 + 0) * Hkv + h) * row, sizeof(uint16_t) * row);
        memcpy(v_pool + dst, tmp + ((size_t)(d * 2 + 1) * Hkv + h) * row, sizeof(uint16_t) * row);
      }
    }
    free(tmp);
    free(path);
    if (new_len) new_len[b] = ctx_len[b] + depth;
  }
  return 0;
}

/* ------------------------------------------------------------------------- */
/* LM head: logits and their per-row softmax statistics                        */
/* ------------------------------------------------------------------------- */
/* Nearest bf16 (ties to even) of a finite double, as its 16 bits.  bf16 carries 8 significant
 * bits; values here are far from its subnormal and overflow ranges. */
static uint16_t double_to_bf16_bits(double x) {
  if (x == 0.0) return signbit(x) ? 0x8000u : 0u;
  int e;
  const double f = frexp(fabs(x), &e);              /* |x| = f * 2^e, f in [0.5, 1) */
  const double q = nearbyint(ldexp(f, 8));          /* 8 significant bits, round half to even */
  const float r = (float)ldexp(q, e - 8);           /* exactly representable */
  uint32_t u;
  memcpy(&u, &r, 4);
  return (uint16_t)((u >> 16) | (signbit(x) ? 0x8000u : 0u));
}

/*
 * hidden [rows, d] bf16, weight [V, d] bf16 (one row per vocabulary entry).
 * exact[r, v]  = sum_k hidden[r, k] * weight[v, k] in fp64 (optional output),
 * logits[r, v] = bf16(exact[r, v]),
 * row_max[r]   = max_v logits[r, v],  row_z[r] = sum_v exp((logits[r, v] - row_max[r]) / T).
 */
int oracle_lm_head(int rows, int d, int V, const uint16_t* hidden, const uint16_t* weight, double T,
                   uint16_t* logits, double* exact, double* row_max, double* row_z) {
  if (rows < 0 || d <= 0 || V <= 0 || !(T > 0.0)) return -2;
#pragma omp parallel for schedule(static)
  for (int r = 0; r < rows; ++r) {
    for (int v = 0; v < V; ++v) {
      double acc = 0.0;
      for (int k = 0; k < d; ++k)
        acc += bf16_to_double(hidden[(int64_t)r * d + k]) * bf16_to_double(weight[(int64_t)v * d + k]);
      if (exact) exact[(int64_t)r * V + v] = acc;
      logits[(int64_t)r * V + v] = double_to_bf16_bits(acc);
    }
    double m = -INFINITY;
    for (int v = 0; v < V; ++v) {
      const double l = bf16_to_double(logits[(int64_t)r * V + v]);
      if (l > m) m = l;
    }
    double z = 0.0;
    for (int v = 0; v < V; ++v) z += exp((bf16_to_double(logits[(int64_t)r * V + v]) - m) / T);
    row_max[r] = m;
    row_z[r] = z;
  }
  return 0;
}
