// CPU oracle for one accelerator's share of a decoder-only Transformer LM train
// step and for the chained-dispatch micro-benchmark.
//
// TEST INFRASTRUCTURE ONLY.  Nothing on the product path may include, link or
// call this file; it exists so that the HIP kernels have an independent,
// obviously correct result to be compared with.  It shares no code with them.
//
// What is computed.  The paper (Section 5.3) describes the workload only in
// words: a decoder-only Transformer language model with an embedding lookup in
// front, a stack of Transformer layers (model dimension d, hidden dimension F)
// and a softmax layer at the end, trained with back-propagation; the step is an
// opaque "compiled function" (Section 3, Appendix B).  The method reaches
// exactly the textbook result, so every function below is the textbook
// definition written as scalar loops: no blocking, no fusion, no reordering.
// OpenMP only splits loops whose iterations are independent.
//
// Readings frozen here where the paper is silent (all are parameters of the
// workload, stated again in the build's design notes):
//   R1  next-token targets: tokens are [B, T+1]; inputs = columns 0..T-1,
//       targets = columns 1..T; loss = mean over all B*T positions.
//   R2  GELU is the tanh form 0.5 u (1 + tanh(sqrt(2/pi) (u + 0.044715 u^3))).
//   R3  LayerNorm: biased variance, rstd = 1/sqrt(var + 1e-5), affine.
//   R4  pre-LayerNorm blocks, one final LayerNorm before the head.
//   R5  untied head Wh [d, V] without bias; biases on QKV, out-proj, FFN1, FFN2.
//   R6  attention scale 1/sqrt(head_dim); position i attends to j <= i; no dropout.
//   R7  learned positional embedding [T, d] added at the input only.
//   R8  SGD: w -= lr g.   Adam: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2;
//       w -= lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps), t counted from 1.
//   R9  weights are [in, out] row-major; Wqkv columns are [Q | K | V]; head h
//       owns columns h*hd .. (h+1)*hd of each third.
//   R10 the dispatch benchmark's "x + L" is L sequential fp32 additions of 1.0f.
//
// Parity pins (tests/test_oracle_pins.py): central finite differences of the
// loss in double for every parameter family; loss = ln V at zero head; softmax
// rows sum to 1, dlogits rows to 0; causal invariance; LayerNorm moments;
// attention closed forms (T=1, Q=0 prefix mean); Adam/SGD closed forms; the
// worked example of the paper's Figure 2.
#pragma once
#include <cmath>
#include <cstdint>
#include <cstring>
#include <string>
#include <vector>

namespace oracle {

// ---- elementwise pieces -------------------------------------------------------------------------

// R2.
template <class S> inline S gelu(S u) {
  const S c = std::sqrt(S(2) / S(M_PI));
  return S(0.5) * u * (S(1) + std::tanh(c * (u + S(0.044715) * u * u * u)));
}
template <class S> inline S gelu_grad(S u) {
  const S c = std::sqrt(S(2) / S(M_PI));
  const S a = c * (u + S(0.044715) * u * u * u);
  const S t = std::tanh(a);
  const S da = c * (S(1) + S(3) * S(0.044715) * u * u);
  return S(0.5) * (S(1) + t) + S(0.5) * u * (S(1) - t * t) * da;
}

// ---- embedding (R1, R7) -------------------------------------------------------------------------

// x[b,t,:] = wte[inp[b,t],:] + wpe[t,:]
template <class S>
void embedding_fwd(const int32_t* inp, const S* wte, const S* wpe, S* x, int B, int T, int d) {
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < T; ++t)
      for (int c = 0; c < d; ++c)
        x[((size_t)b * T + t) * d + c] = wte[(size_t)inp[b * T + t] * d + c] + wpe[(size_t)t * d + c];
}

// dwte[inp[b,t],:] += dx[b,t,:] (equal ids accumulate);  dwpe[t,:] = sum_b dx[b,t,:]
template <class S>
void embedding_bwd(const int32_t* inp, const S* dx, S* dwte, S* dwpe, int B, int T, int d, int V) {
  std::fill(dwte, dwte + (size_t)V * d, S(0));
  std::fill(dwpe, dwpe + (size_t)T * d, S(0));
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < T; ++t)
      for (int c = 0; c < d; ++c) {
        const S g = dx[((size_t)b * T + t) * d + c];
        dwte[(size_t)inp[b * T + t] * d + c] += g;
        dwpe[(size_t)t * d + c] += g;
      }
}

// ---- LayerNorm (R3) -----------------------------------------------------------------------------

template <class S>
void layernorm_fwd(const S* x, const S* g, const S* b, S* y, S* mean, S* rstd, int N, int d) {
#pragma omp parallel for
  for (int n = 0; n < N; ++n) {
    const S* xr = x + (size_t)n * d;
    S mu = 0;
    for (int c = 0; c < d; ++c) mu += xr[c];
    mu /= S(d);
    S var = 0;
    for (int c = 0; c < d; ++c) var += (xr[c] - mu) * (xr[c] - mu);
    var /= S(d);
    const S rs = S(1) / std::sqrt(var + S(1e-5));
    for (int c = 0; c < d; ++c) y[(size_t)n * d + c] = (xr[c] - mu) * rs * g[c] + b[c];
    if (mean) mean[n] = mu;
    if (rstd) rstd[n] = rs;
  }
}

// With xh = (x - mean) rstd and gg = dy*g:  dx = rstd (gg - mean_c(gg) - xh mean_c(gg xh));
// dg = sum_n dy xh;  db = sum_n dy.
template <class S>
void layernorm_bwd(const S* dy, const S* x, const S* g, S* dx, S* dg, S* db, int N, int d) {
  std::fill(dg, dg + d, S(0));
  std::fill(db, db + d, S(0));
  for (int n = 0; n < N; ++n) {
    const S* xr = x + (size_t)n * d;
    const S* dyr = dy + (size_t)n * d;
    S mu = 0;
    for (int c = 0; c < d; ++c) mu += xr[c];
    mu /= S(d);
    S var = 0;
    for (int c = 0; c < d; ++c) var += (xr[c] - mu) * (xr[c] - mu);
    var /= S(d);
    const S rs = S(1) / std::sqrt(var + S(1e-5));
    S m1 = 0, m2 = 0;
    for (int c = 0; c < d; ++c) {
      const S xh = (xr[c] - mu) * rs;
      m1 += dyr[c] * g[c];
      m2 += dyr[c] * g[c] * xh;
    }
    m1 /= S(d);
    m2 /= S(d);
    for (int c = 0; c < d; ++c) {
      const S xh = (xr[c] - mu) * rs;
      dx[(size_t)n * d + c] = rs * (dyr[c] * g[c] - m1 - xh * m2);
      dg[c] += dyr[c] * xh;
      db[c] += dyr[c];
    }
  }
}

// ---- linear (R9) --------------------------------------------------------------------------------

// y[n,o] = sum_i x[n,i] W[i,o] (+ b[o])
template <class S>
void linear_fwd(const S* x, const S* W, const S* b, S* y, int N, int in, int out) {
#pragma omp parallel for
  for (int n = 0; n < N; ++n) {
    S* yr = y + (size_t)n * out;
    for (int o = 0; o < out; ++o) yr[o] = b ? b[o] : S(0);
    for (int i = 0; i < in; ++i) {
      const S xi = x[(size_t)n * in + i];
      const S* wr = W + (size_t)i * out;
      for (int o = 0; o < out; ++o) yr[o] += xi * wr[o];
    }
  }
}

// dx[n,i] = sum_o dy[n,o] W[i,o];  dW[i,o] = sum_n x[n,i] dy[n,o];  db[o] = sum_n dy[n,o]
template <class S>
void linear_bwd(const S* x, const S* W, const S* dy, S* dx, S* dW, S* db, int N, int in, int out) {
  if (dx) {
#pragma omp parallel for
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < in; ++i) {
        S acc = 0;
        for (int o = 0; o < out; ++o) acc += dy[(size_t)n * out + o] * W[(size_t)i * out + o];
        dx[(size_t)n * in + i] = acc;
      }
  }
  if (dW) {
#pragma omp parallel for
    for (int i = 0; i < in; ++i) {
      S* dwr = dW + (size_t)i * out;
      for (int o = 0; o < out; ++o) dwr[o] = 0;
      for (int n = 0; n < N; ++n) {
        const S xi = x[(size_t)n * in + i];
        const S* dyr = dy + (size_t)n * out;
        for (int o = 0; o < out; ++o) dwr[o] += xi * dyr[o];
      }
    }
  }
  if (db) {
    for (int o = 0; o < out; ++o) db[o] = 0;
    for (int n = 0; n < N; ++n)
      for (int o = 0; o < out; ++o) db[o] += dy[(size_t)n * out + o];
  }
}

// ---- causal multi-head attention (R6, R9) -------------------------------------------------------

// qkv is [B*T, 3d]: q_i = qkv[row i, h*hd ..], k_j = qkv[row j, d + h*hd ..], v_j = qkv[row j, 2d + h*hd ..].
// Fills p[j] = softmax_{j<=i}(q_i.k_j / sqrt(hd)) for one (b, h, i).
template <class S>
void attention_probs_row(const S* qkv, int b, int h, int i, int T, int d, int hd, S* p) {
  const S scale = S(1) / std::sqrt(S(hd));
  const S* q = qkv + ((size_t)b * T + i) * 3 * d + (size_t)h * hd;
  S mx = -INFINITY;
  for (int j = 0; j <= i; ++j) {
    const S* k = qkv + ((size_t)b * T + j) * 3 * d + d + (size_t)h * hd;
    S s = 0;
    for (int c = 0; c < hd; ++c) s += q[c] * k[c];
    p[j] = s * scale;
    if (p[j] > mx) mx = p[j];
  }
  S sum = 0;
  for (int j = 0; j <= i; ++j) {
    p[j] = std::exp(p[j] - mx);
    sum += p[j];
  }
  for (int j = 0; j <= i; ++j) p[j] /= sum;
}

// o[b,i,h*hd+c] = sum_{j<=i} p[i,j] v[j,c].  probs (optional) receives [B,H,T,T], zeros above the diagonal.
template <class S>
void attention_fwd(const S* qkv, S* o, S* probs, int B, int T, int H, int hd) {
  const int d = H * hd;
#pragma omp parallel for collapse(2)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      std::vector<S> p(T);
      for (int i = 0; i < T; ++i) {
        attention_probs_row(qkv, b, h, i, T, d, hd, p.data());
        S* orow = o + ((size_t)b * T + i) * d + (size_t)h * hd;
        for (int c = 0; c < hd; ++c) orow[c] = 0;
        for (int j = 0; j <= i; ++j) {
          const S* v = qkv + ((size_t)b * T + j) * 3 * d + 2 * d + (size_t)h * hd;
          for (int c = 0; c < hd; ++c) orow[c] += p[j] * v[c];
        }
        if (probs) {
          S* pr = probs + (((size_t)b * H + h) * T + i) * T;
          for (int j = 0; j < T; ++j) pr[j] = j <= i ? p[j] : S(0);
        }
      }
    }
}

// dv_j = sum_{i>=j} p_ij do_i;  dp_ij = do_i.v_j;  ds_ij = p_ij (dp_ij - sum_k p_ik dp_ik);
// dq_i = sum_{j<=i} ds_ij k_j / sqrt(hd);  dk_j = sum_{i>=j} ds_ij q_i / sqrt(hd).
template <class S>
void attention_bwd(const S* qkv, const S* dout, S* dqkv, int B, int T, int H, int hd) {
  const int d = H * hd;
  const S scale = S(1) / std::sqrt(S(hd));
  std::fill(dqkv, dqkv + (size_t)B * T * 3 * d, S(0));
#pragma omp parallel for collapse(2)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      std::vector<S> p(T), dp(T);
      for (int i = 0; i < T; ++i) {
        attention_probs_row(qkv, b, h, i, T, d, hd, p.data());
        const S* q = qkv + ((size_t)b * T + i) * 3 * d + (size_t)h * hd;
        const S* go = dout + ((size_t)b * T + i) * d + (size_t)h * hd;
        S* dq = dqkv + ((size_t)b * T + i) * 3 * d + (size_t)h * hd;
        S dot = 0;
        for (int j = 0; j <= i; ++j) {
          const S* v = qkv + ((size_t)b * T + j) * 3 * d + 2 * d + (size_t)h * hd;
          S a = 0;
          for (int c = 0; c < hd; ++c) a += go[c] * v[c];
          dp[j] = a;
          dot += p[j] * a;
        }
        for (int j = 0; j <= i; ++j) {
          const S ds = p[j] * (dp[j] - dot);
          const S* k = qkv + ((size_t)b * T + j) * 3 * d + d + (size_t)h * hd;
          S* dk = dqkv + ((size_t)b * T + j) * 3 * d + d + (size_t)h * hd;
          S* dv = dqkv + ((size_t)b * T + j) * 3 * d + 2 * d + (size_t)h * hd;
          for (int c = 0; c < hd; ++c) {
            dq[c] += ds * k[c] * scale;
            dk[c] += ds * q[c] * scale;
            dv[c] += p[j] * go[c];
          }
        }
      }
    }
}

// ---- softmax cross-entropy (R1) -----------------------------------------------------------------

// loss = (1/N) sum_n [ log sum_v exp(z[n,v]) - z[n,tgt[n]] ];  dz = (softmax(z) - onehot(tgt)) / N.
template <class S>
void softmax_xent(const S* z, const int32_t* tgt, int N, int V, S* loss, S* dz) {
  std::vector<S> row_loss(N);
#pragma omp parallel for
  for (int n = 0; n < N; ++n) {
    const S* zr = z + (size_t)n * V;
    S mx = zr[0];
    for (int v = 1; v < V; ++v) mx = zr[v] > mx ? zr[v] : mx;
    S sum = 0;
    for (int v = 0; v < V; ++v) sum += std::exp(zr[v] - mx);
    row_loss[n] = std::log(sum) + mx - zr[tgt[n]];
    if (dz) {
      S* dr = dz + (size_t)n * V;
      for (int v = 0; v < V; ++v) dr[v] = std::exp(zr[v] - mx) / sum / S(N);
      dr[tgt[n]] -= S(1) / S(N);
    }
  }
  S total = 0;
  for (int n = 0; n < N; ++n) total += row_loss[n];
  *loss = total / S(N);
}

// ---- optimisers (R8) ----------------------------------------------------------------------------

template <class S> void sgd(S* w, const S* g, size_t n, S lr) {
  for (size_t i = 0; i < n; ++i) w[i] -= lr * g[i];
}

template <class S>
void adam(S* w, S* m, S* v, const S* g, size_t n, S lr, S b1, S b2, S eps, int t) {
  const S c1 = S(1) - std::pow(b1, S(t));
  const S c2 = S(1) - std::pow(b2, S(t));
  for (size_t i = 0; i < n; ++i) {
    m[i] = b1 * m[i] + (S(1) - b1) * g[i];
    v[i] = b2 * v[i] + (S(1) - b2) * g[i] * g[i];
    w[i] -= lr * (m[i] / c1) / (std::sqrt(v[i] / c2) + eps);
  }
}

// ---- whole model --------------------------------------------------------------------------------

struct LMShape {
  int L, d, H, F, V, T, B;
  int has_embed, has_head;   // a pipeline stage has neither
};

struct ParamEntry {
  std::string name;
  size_t offset, numel;
};

// Flat parameter vector of this oracle (its own layout; callers marshal by name).
inline std::vector<ParamEntry> param_table(const LMShape& s) {
  std::vector<ParamEntry> t;
  size_t off = 0;
  auto add = [&](const std::string& n, size_t numel) {
    t.push_back({n, off, numel});
    off += numel;
  };
  const size_t d = s.d, F = s.F, V = s.V, T = s.T;
  if (s.has_embed) {
    add("wte", V * d);
    add("wpe", T * d);
  }
  for (int l = 0; l < s.L; ++l) {
    const std::string p = "l" + std::to_string(l) + ".";
    add(p + "ln1_g", d); add(p + "ln1_b", d);
    add(p + "wqkv", d * 3 * d); add(p + "bqkv", 3 * d);
    add(p + "wo", d * d); add(p + "bo", d);
    add(p + "ln2_g", d); add(p + "ln2_b", d);
    add(p + "w1", d * F); add(p + "b1", F);
    add(p + "w2", F * d); add(p + "b2", d);
  }
  if (s.has_head) {
    add("lnf_g", d); add("lnf_b", d);
    add("wh", d * V);
  }
  return t;
}

inline size_t param_total(const LMShape& s) {
  auto t = param_table(s);
  return t.empty() ? 0 : t.back().offset + t.back().numel;
}

template <class S> struct LayerActs {
  std::vector<S> x_in, a, qkv, o, x_mid, m, u, h;
};

// Forward and (optionally) backward through the layer stack, R4 block structure:
//   x_mid = x_in + attn(LN1(x_in)) Wo + bo ;  x_out = x_mid + gelu(LN2(x_mid) W1 + b1) W2 + b2.
// `x0` is the stack input [N, d]; on return `x_out` holds the stack output.
template <class S>
void layers_fwd(const LMShape& s, const S* P, const std::vector<ParamEntry>& tab, size_t first,
                const S* x0, std::vector<LayerActs<S>>& acts, std::vector<S>& x_out) {
  const int N = s.B * s.T, d = s.d, F = s.F, hd = s.d / s.H;
  std::vector<S> x(x0, x0 + (size_t)N * d);
  acts.resize(s.L);
  for (int l = 0; l < s.L; ++l) {
    const size_t e = first + (size_t)l * 12;
    const S *ln1g = P + tab[e].offset, *ln1b = P + tab[e + 1].offset, *wqkv = P + tab[e + 2].offset,
            *bqkv = P + tab[e + 3].offset, *wo = P + tab[e + 4].offset, *bo = P + tab[e + 5].offset,
            *ln2g = P + tab[e + 6].offset, *ln2b = P + tab[e + 7].offset, *w1 = P + tab[e + 8].offset,
            *b1 = P + tab[e + 9].offset, *w2 = P + tab[e + 10].offset, *b2 = P + tab[e + 11].offset;
    LayerActs<S>& A = acts[l];
    A.x_in = x;
    A.a.resize((size_t)N * d);
    layernorm_fwd<S>(x.data(), ln1g, ln1b, A.a.data(), nullptr, nullptr, N, d);
    A.qkv.resize((size_t)N * 3 * d);
    linear_fwd<S>(A.a.data(), wqkv, bqkv, A.qkv.data(), N, d, 3 * d);
    A.o.resize((size_t)N * d);
    attention_fwd<S>(A.qkv.data(), A.o.data(), nullptr, s.B, s.T, s.H, hd);
    std::vector<S> proj((size_t)N * d);
    linear_fwd<S>(A.o.data(), wo, bo, proj.data(), N, d, d);
    for (size_t i = 0; i < x.size(); ++i) x[i] += proj[i];
    A.x_mid = x;
    A.m.resize((size_t)N * d);
    layernorm_fwd<S>(x.data(), ln2g, ln2b, A.m.data(), nullptr, nullptr, N, d);
    A.u.resize((size_t)N * F);
    linear_fwd<S>(A.m.data(), w1, b1, A.u.data(), N, d, F);
    A.h.resize((size_t)N * F);
    for (size_t i = 0; i < A.u.size(); ++i) A.h[i] = gelu<S>(A.u[i]);
    linear_fwd<S>(A.h.data(), w2, b2, proj.data(), N, F, d);
    for (size_t i = 0; i < x.size(); ++i) x[i] += proj[i];
  }
  x_out = x;
}

// dx (in: gradient w.r.t. the stack output; out: w.r.t. the stack input).  Parameter gradients are
// ADDED into G (so a pipeline stage can accumulate over micro-batches); callers zero G first.
template <class S>
void layers_bwd(const LMShape& s, const S* P, S* G, const std::vector<ParamEntry>& tab, size_t first,
                const std::vector<LayerActs<S>>& acts, std::vector<S>& dx) {
  const int N = s.B * s.T, d = s.d, F = s.F, hd = s.d / s.H;
  auto accum = [&](size_t entry, const std::vector<S>& g) {
    S* dst = G + tab[entry].offset;
    for (size_t i = 0; i < g.size(); ++i) dst[i] += g[i];
  };
  for (int l = s.L - 1; l >= 0; --l) {
    const size_t e = first + (size_t)l * 12;
    const S *ln1g = P + tab[e].offset, *wqkv = P + tab[e + 2].offset, *wo = P + tab[e + 4].offset,
            *ln2g = P + tab[e + 6].offset, *w1 = P + tab[e + 8].offset, *w2 = P + tab[e + 10].offset;
    const LayerActs<S>& A = acts[l];
    // x_out = x_mid + h W2 + b2
    std::vector<S> dh((size_t)N * F), dW2((size_t)F * d), db2(d);
    linear_bwd<S>(A.h.data(), w2, dx.data(), dh.data(), dW2.data(), db2.data(), N, F, d);
    accum(e + 10, dW2); accum(e + 11, db2);
    std::vector<S> du((size_t)N * F);
    for (size_t i = 0; i < du.size(); ++i) du[i] = dh[i] * gelu_grad<S>(A.u[i]);
    std::vector<S> dm((size_t)N * d), dW1((size_t)d * F), db1(F);
    linear_bwd<S>(A.m.data(), w1, du.data(), dm.data(), dW1.data(), db1.data(), N, d, F);
    accum(e + 8, dW1); accum(e + 9, db1);
    std::vector<S> dxl((size_t)N * d), dg(d), dbeta(d);
    layernorm_bwd<S>(dm.data(), A.x_mid.data(), ln2g, dxl.data(), dg.data(), dbeta.data(), N, d);
    accum(e + 6, dg); accum(e + 7, dbeta);
    for (size_t i = 0; i < dx.size(); ++i) dx[i] += dxl[i];   // residual: both branches sum
    // x_mid = x_in + o Wo + bo
    std::vector<S> dO((size_t)N * d), dWo((size_t)d * d), dbo(d);
    linear_bwd<S>(A.o.data(), wo, dx.data(), dO.data(), dWo.data(), dbo.data(), N, d, d);
    accum(e + 4, dWo); accum(e + 5, dbo);
    std::vector<S> dqkv((size_t)N * 3 * d);
    attention_bwd<S>(A.qkv.data(), dO.data(), dqkv.data(), s.B, s.T, s.H, hd);
    std::vector<S> da((size_t)N * d), dWqkv((size_t)d * 3 * d), dbqkv(3 * d);
    linear_bwd<S>(A.a.data(), wqkv, dqkv.data(), da.data(), dWqkv.data(), dbqkv.data(), N, d, 3 * d);
    accum(e + 2, dWqkv); accum(e + 3, dbqkv);
    layernorm_bwd<S>(da.data(), A.x_in.data(), ln1g, dxl.data(), dg.data(), dbeta.data(), N, d);
    accum(e, dg); accum(e + 1, dbeta);
    for (size_t i = 0; i < dx.size(); ++i) dx[i] += dxl[i];
  }
}

struct OptConfig {
  int kind;   // 0 none, 1 SGD, 2 Adam
  double lr, beta1, beta2, eps;
  int t;      // Adam step number, from 1
};

// One full train step of the LM (embedding .. head .. loss, backward, update).  P is updated in place
// when opt.kind != 0; G receives the gradients; logits (optional) [N, V]; do_bwd = 0 stops after the loss.
template <class S>
void lm_train_step(const LMShape& s, S* P, S* M, S* Vv, const int32_t* tokens, const OptConfig& opt,
                   S* loss, S* G, S* logits, int do_bwd) {
  const int N = s.B * s.T, d = s.d, V = s.V, T = s.T;
  const auto tab = param_table(s);
  const size_t total = param_total(s);
  std::vector<int32_t> inp(N), tgt(N);
  for (int b = 0; b < s.B; ++b)
    for (int t = 0; t < T; ++t) {
      inp[b * T + t] = tokens[b * (T + 1) + t];
      tgt[b * T + t] = tokens[b * (T + 1) + t + 1];
    }
  const S *wte = P + tab[0].offset, *wpe = P + tab[1].offset;
  const size_t first = 2, tail = 2 + (size_t)s.L * 12;
  const S *lnfg = P + tab[tail].offset, *lnfb = P + tab[tail + 1].offset, *wh = P + tab[tail + 2].offset;

  std::vector<S> x0((size_t)N * d), xL;
  embedding_fwd<S>(inp.data(), wte, wpe, x0.data(), s.B, T, d);
  std::vector<LayerActs<S>> acts;
  layers_fwd<S>(s, P, tab, first, x0.data(), acts, xL);
  std::vector<S> y((size_t)N * d), z((size_t)N * V);
  layernorm_fwd<S>(xL.data(), lnfg, lnfb, y.data(), nullptr, nullptr, N, d);
  linear_fwd<S>(y.data(), wh, nullptr, z.data(), N, d, V);
  if (logits) std::memcpy(logits, z.data(), z.size() * sizeof(S));
  std::vector<S> dz(do_bwd ? z.size() : 0);
  softmax_xent<S>(z.data(), tgt.data(), N, V, loss, do_bwd ? dz.data() : nullptr);
  if (!do_bwd) return;

  std::fill(G, G + total, S(0));
  std::vector<S> dy((size_t)N * d);
  linear_bwd<S>(y.data(), wh, dz.data(), dy.data(), G + tab[tail + 2].offset, nullptr, N, d, V);
  std::vector<S> dx((size_t)N * d);
  layernorm_bwd<S>(dy.data(), xL.data(), lnfg, dx.data(), G + tab[tail].offset, G + tab[tail + 1].offset, N, d);
  layers_bwd<S>(s, P, G, tab, first, acts, dx);
  embedding_bwd<S>(inp.data(), dx.data(), G + tab[0].offset, G + tab[1].offset, s.B, T, d, V);

  if (opt.kind == 1) sgd<S>(P, G, total, S(opt.lr));
  if (opt.kind == 2) adam<S>(P, M, Vv, G, total, S(opt.lr), S(opt.beta1), S(opt.beta2), S(opt.eps), opt.t);
}

// One pipeline stage under the GPipe-like schedule of Section 5.3: forward for every micro-batch in
// order, then backward in reverse order, parameter gradients summed over micro-batches.
// X, dY: [n_mb][N, d] inputs; Y, dX: [n_mb][N, d] outputs; G: summed gradients.
template <class S>
void stage_fwd_bwd(const LMShape& s, const S* P, int n_mb, const S* X, const S* dY, S* Y, S* dX, S* G) {
  const size_t N = (size_t)s.B * s.T, d = s.d;
  const auto tab = param_table(s);
  std::fill(G, G + param_total(s), S(0));
  std::vector<std::vector<LayerActs<S>>> stash(n_mb);
  for (int mb = 0; mb < n_mb; ++mb) {
    std::vector<S> out;
    layers_fwd<S>(s, P, tab, 0, X + mb * N * d, stash[mb], out);
    std::memcpy(Y + mb * N * d, out.data(), N * d * sizeof(S));
  }
  for (int mb = n_mb - 1; mb >= 0; --mb) {
    std::vector<S> dx(dY + mb * N * d, dY + (mb + 1) * N * d);
    layers_bwd<S>(s, P, G, tab, 0, stash[mb], dx);
    std::memcpy(dX + mb * N * d, dx.data(), N * d * sizeof(S));
  }
}

// ---- dispatch micro-benchmark (Section 5.1; R10) ------------------------------------------------

// The chained function of the benchmark: y = x + c in fp32, applied L times in sequence.
inline void chain_add_f32(const float* x, float* y, int n, int L, float c) {
  for (int i = 0; i < n; ++i) {
    volatile float acc = x[i];
    for (int k = 0; k < L; ++k) acc = acc + c;
    y[i] = acc;
  }
}

// The three compiled functions of the paper's Figure 2, in fp32: kind 0: x*c, 1: x+c, 2: x/c.
inline void scalar_fn_f32(int kind, const float* x, float* y, int n, float c) {
  for (int i = 0; i < n; ++i) y[i] = kind == 0 ? x[i] * c : kind == 1 ? x[i] + c : x[i] / c;
}

}  // namespace oracle
