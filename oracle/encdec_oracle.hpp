// CPU oracle, second workload: one accelerator's share of an encoder-decoder Transformer train step.
//
// TEST INFRASTRUCTURE ONLY, like lm_oracle.hpp, whose pieces (LayerNorm, linear, GELU, embedding,
// softmax cross-entropy, optimisers) it reuses.  It shares no code with the HIP path.
//
// What is computed.  The paper's Table 1 measures training throughput of text-to-text
// encoder-decoder Transformers of four sizes; its text gives neither their layer recipe nor their
// hyper-parameters.  The workload here keeps what defines that family - an encoder stack whose
// attention sees the whole source, a decoder stack with causal self-attention plus attention over
// the encoder's output, next-token loss on the target side - and builds it from the pieces the
// decoder-only model already fixed (readings R2..R9 of lm_oracle.hpp).  Every function is the
// textbook definition as scalar loops.
//
// Readings frozen here (the paper is silent on all of them):
//   E1 source tokens are [B, Ts], all visible to every encoder position; target tokens are
//       [B, Tt+1]: decoder inputs = columns 0..Tt-1, targets = columns 1..Tt; loss = mean over the
//       B*Tt target positions.
//   E2 encoder layer: x += SelfAttn_full(LN1 x) Wo + bo;  x += FFN(LN2 x).
//       decoder layer: y += SelfAttn_causal(LN1 y) Wo + bo;  y += CrossAttn(LNx y, mem) Wox + box;
//       y += FFN(LN2 y).  mem = LNf_enc(encoder stack output); logits = LNf_dec(y) Wh.
//   E3 cross-attention: queries q = LNx(y) Wq + bq from the decoder, keys and values
//       [K | V] = mem Wkv + bkv from the encoder output, scale 1/sqrt(head_dim), no mask.
//   E4 encoder and decoder have their own token and position tables; the head is untied.
//
// Parity pins (tests/test_oracle_pins_encdec.py): attention closed forms without a mask (zero queries give
// the mean of all values; one key returns its value; key order does not matter); agreement with a
// softmax written with library routines; central finite differences of the loss for every parameter
// family; with Wox = box = 0 the decoder is the pinned decoder-only model, loss and gradients; a
// permutation of the source positions applied to tokens and position table alike leaves the loss
// unchanged.
#pragma once
#include "lm_oracle.hpp"

namespace oracle {

// ---- multi-head attention of Tq queries over Tk keys (R6, E3) -----------------------------------

// q, k, v point at (batch 0, row 0, feature 0); rows are ldq (q) / ldkv (k, v) elements apart, batch b
// starts at row b*Tq (q) / b*Tk (k, v); head h owns features h*hd .. (h+1)*hd of a row.
// causal != 0: query i sees keys j <= i (callers pass Tq == Tk).  p[j] over the visible keys.
template <class S>
int mha_probs_row(const S* q, size_t ldq, const S* k, size_t ldkv, int b, int h, int i, int Tq, int Tk, int hd,
                  int causal, S* p) {
  const S scale = S(1) / std::sqrt(S(hd));
  const int n = causal ? i + 1 : Tk;
  const S* qi = q + ((size_t)b * Tq + i) * ldq + (size_t)h * hd;
  S mx = -INFINITY;
  for (int j = 0; j < n; ++j) {
    const S* kj = k + ((size_t)b * Tk + j) * ldkv + (size_t)h * hd;
    S s = 0;
    for (int c = 0; c < hd; ++c) s += qi[c] * kj[c];
    p[j] = s * scale;
    if (p[j] > mx) mx = p[j];
  }
  S sum = 0;
  for (int j = 0; j < n; ++j) {
    p[j] = std::exp(p[j] - mx);
    sum += p[j];
  }
  for (int j = 0; j < n; ++j) p[j] /= sum;
  return n;
}

// o[b*Tq+i, h*hd+c] = sum_j p_ij v[j, c];  o is dense [B*Tq, H*hd].
template <class S>
void mha_fwd(const S* q, size_t ldq, const S* k, const S* v, size_t ldkv, S* o, int B, int Tq, int Tk, int H,
             int hd, int causal) {
  const size_t d = (size_t)H * hd;
#pragma omp parallel for collapse(2)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      std::vector<S> p(Tk);
      for (int i = 0; i < Tq; ++i) {
        const int n = mha_probs_row(q, ldq, k, ldkv, b, h, i, Tq, Tk, hd, causal, p.data());
        S* orow = o + ((size_t)b * Tq + i) * d + (size_t)h * hd;
        for (int c = 0; c < hd; ++c) orow[c] = 0;
        for (int j = 0; j < n; ++j) {
          const S* vj = v + ((size_t)b * Tk + j) * ldkv + (size_t)h * hd;
          for (int c = 0; c < hd; ++c) orow[c] += p[j] * vj[c];
        }
      }
    }
}

// dv_j = sum_i p_ij do_i;  dp_ij = do_i.v_j;  ds_ij = p_ij (dp_ij - sum_k p_ik dp_ik);
// dq_i = sum_j ds_ij k_j / sqrt(hd);  dk_j = sum_i ds_ij q_i / sqrt(hd)   (sums over visible pairs).
// dq rows are lddq apart, dk and dv rows lddkv; the H*hd features of every row are overwritten.
template <class S>
void mha_bwd(const S* q, size_t ldq, const S* k, const S* v, size_t ldkv, const S* dout, S* dq, size_t lddq, S* dk,
             S* dv, size_t lddkv, int B, int Tq, int Tk, int H, int hd, int causal) {
  const size_t d = (size_t)H * hd;
  const S scale = S(1) / std::sqrt(S(hd));
  for (size_t r = 0; r < (size_t)B * Tq; ++r) std::fill(dq + r * lddq, dq + r * lddq + d, S(0));
  for (size_t r = 0; r < (size_t)B * Tk; ++r) {
    std::fill(dk + r * lddkv, dk + r * lddkv + d, S(0));
    std::fill(dv + r * lddkv, dv + r * lddkv + d, S(0));
  }
#pragma omp parallel for collapse(2)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      std::vector<S> p(Tk), dp(Tk);
      for (int i = 0; i < Tq; ++i) {
        const int n = mha_probs_row(q, ldq, k, ldkv, b, h, i, Tq, Tk, hd, causal, p.data());
        const S* qi = q + ((size_t)b * Tq + i) * ldq + (size_t)h * hd;
        const S* go = dout + ((size_t)b * Tq + i) * d + (size_t)h * hd;
        S* dqi = dq + ((size_t)b * Tq + i) * lddq + (size_t)h * hd;
        S dot = 0;
        for (int j = 0; j < n; ++j) {
          const S* vj = v + ((size_t)b * Tk + j) * ldkv + (size_t)h * hd;
          S a = 0;
          for (int c = 0; c < hd; ++c) a += go[c] * vj[c];
          dp[j] = a;
          dot += p[j] * a;
        }
        for (int j = 0; j < n; ++j) {
          const S ds = p[j] * (dp[j] - dot);
          const S* kj = k + ((size_t)b * Tk + j) * ldkv + (size_t)h * hd;
          S* dkj = dk + ((size_t)b * Tk + j) * lddkv + (size_t)h * hd;
          S* dvj = dv + ((size_t)b * Tk + j) * lddkv + (size_t)h * hd;
          for (int c = 0; c < hd; ++c) {
            dqi[c] += ds * kj[c] * scale;
            dkj[c] += ds * qi[c] * scale;
            dvj[c] += p[j] * go[c];
          }
        }
      }
    }
}

// ---- the model ----------------------------------------------------------------------------------

struct EncDecShape {
  int Le, Ld, d, H, F, V, Ts, Tt, B;
};

constexpr size_t kEncLayerParams = 12, kDecLayerParams = 20;

// Flat parameter vector of this oracle (its own layout; callers marshal by name).
inline std::vector<ParamEntry> encdec_param_table(const EncDecShape& s) {
  std::vector<ParamEntry> t;
  size_t off = 0;
  auto add = [&](const std::string& n, size_t numel) {
    t.push_back({n, off, numel});
    off += numel;
  };
  const size_t d = s.d, F = s.F, V = s.V;
  add("enc.wte", V * d);
  add("enc.wpe", (size_t)s.Ts * d);
  for (int l = 0; l < s.Le; ++l) {
    const std::string p = "e" + std::to_string(l) + ".";
    add(p + "ln1_g", d); add(p + "ln1_b", d);
    add(p + "wqkv", d * 3 * d); add(p + "bqkv", 3 * d);
    add(p + "wo", d * d); add(p + "bo", d);
    add(p + "ln2_g", d); add(p + "ln2_b", d);
    add(p + "w1", d * F); add(p + "b1", F);
    add(p + "w2", F * d); add(p + "b2", d);
  }
  add("enc.lnf_g", d); add("enc.lnf_b", d);
  add("dec.wte", V * d);
  add("dec.wpe", (size_t)s.Tt * d);
  for (int l = 0; l < s.Ld; ++l) {
    const std::string p = "d" + std::to_string(l) + ".";
    add(p + "ln1_g", d); add(p + "ln1_b", d);
    add(p + "wqkv", d * 3 * d); add(p + "bqkv", 3 * d);
    add(p + "wo", d * d); add(p + "bo", d);
    add(p + "lnx_g", d); add(p + "lnx_b", d);
    add(p + "wq", d * d); add(p + "bq", d);
    add(p + "wkv", d * 2 * d); add(p + "bkv", 2 * d);
    add(p + "wox", d * d); add(p + "box", d);
    add(p + "ln2_g", d); add(p + "ln2_b", d);
    add(p + "w1", d * F); add(p + "b1", F);
    add(p + "w2", F * d); add(p + "b2", d);
  }
  add("dec.lnf_g", d); add("dec.lnf_b", d);
  add("wh", d * V);
  return t;
}

inline size_t encdec_param_total(const EncDecShape& s) {
  auto t = encdec_param_table(s);
  return t.back().offset + t.back().numel;
}

// One residual sub-block remembers its input and what its backward pass needs.
template <class S> struct SelfActs { std::vector<S> x_in, a, qkv, o; };
template <class S> struct CrossActs { std::vector<S> x_in, a, q, kv, o; };
template <class S> struct FfnActs { std::vector<S> x_in, m, u, h; };

// x += Attn(LN(x) Wqkv + bqkv) Wo + bo over T positions per batch; params at tab[e .. e+5].
template <class S>
void self_block_fwd(const S* P, const std::vector<ParamEntry>& tab, size_t e, std::vector<S>& x, SelfActs<S>& A,
                    int B, int T, int d, int H, int causal) {
  const int N = B * T;
  A.x_in = x;
  A.a.resize((size_t)N * d);
  layernorm_fwd<S>(x.data(), P + tab[e].offset, P + tab[e + 1].offset, A.a.data(), nullptr, nullptr, N, d);
  A.qkv.resize((size_t)N * 3 * d);
  linear_fwd<S>(A.a.data(), P + tab[e + 2].offset, P + tab[e + 3].offset, A.qkv.data(), N, d, 3 * d);
  A.o.resize((size_t)N * d);
  mha_fwd<S>(A.qkv.data(), 3 * (size_t)d, A.qkv.data() + d, A.qkv.data() + 2 * d, 3 * (size_t)d, A.o.data(), B, T, T,
             H, d / H, causal);
  std::vector<S> proj((size_t)N * d);
  linear_fwd<S>(A.o.data(), P + tab[e + 4].offset, P + tab[e + 5].offset, proj.data(), N, d, d);
  for (size_t i = 0; i < x.size(); ++i) x[i] += proj[i];
}

// dx: gradient w.r.t. the sub-block's output on entry, w.r.t. its input on return.
template <class S>
void self_block_bwd(const S* P, S* G, const std::vector<ParamEntry>& tab, size_t e, const SelfActs<S>& A,
                    std::vector<S>& dx, int B, int T, int d, int H, int causal) {
  const int N = B * T;
  std::vector<S> dO((size_t)N * d);
  linear_bwd<S>(A.o.data(), P + tab[e + 4].offset, dx.data(), dO.data(), G + tab[e + 4].offset, G + tab[e + 5].offset, N, d, d);
  std::vector<S> dqkv((size_t)N * 3 * d);
  mha_bwd<S>(A.qkv.data(), 3 * (size_t)d, A.qkv.data() + d, A.qkv.data() + 2 * d, 3 * (size_t)d, dO.data(), dqkv.data(),
             3 * (size_t)d, dqkv.data() + d, dqkv.data() + 2 * d, 3 * (size_t)d, B, T, T, H, d / H, causal);
  std::vector<S> da((size_t)N * d);
  linear_bwd<S>(A.a.data(), P + tab[e + 2].offset, dqkv.data(), da.data(), G + tab[e + 2].offset, G + tab[e + 3].offset, N, d, 3 * d);
  std::vector<S> dxl((size_t)N * d);
  layernorm_bwd<S>(da.data(), A.x_in.data(), P + tab[e].offset, dxl.data(), G + tab[e].offset, G + tab[e + 1].offset, N, d);
  for (size_t i = 0; i < dx.size(); ++i) dx[i] += dxl[i];   // residual: both branches sum
}

// y += Attn(q = LN(y) Wq + bq; [K|V] = mem Wkv + bkv) Wox + box; params at tab[e .. e+7]
// (lnx_g, lnx_b, wq, bq, wkv, bkv, wox, box).
template <class S>
void cross_block_fwd(const S* P, const std::vector<ParamEntry>& tab, size_t e, std::vector<S>& y,
                     const std::vector<S>& mem, CrossActs<S>& A, int B, int Tt, int Ts, int d, int H) {
  const int N = B * Tt, Ns = B * Ts;
  A.x_in = y;
  A.a.resize((size_t)N * d);
  layernorm_fwd<S>(y.data(), P + tab[e].offset, P + tab[e + 1].offset, A.a.data(), nullptr, nullptr, N, d);
  A.q.resize((size_t)N * d);
  linear_fwd<S>(A.a.data(), P + tab[e + 2].offset, P + tab[e + 3].offset, A.q.data(), N, d, d);
  A.kv.resize((size_t)Ns * 2 * d);
  linear_fwd<S>(mem.data(), P + tab[e + 4].offset, P + tab[e + 5].offset, A.kv.data(), Ns, d, 2 * d);
  A.o.resize((size_t)N * d);
  mha_fwd<S>(A.q.data(), (size_t)d, A.kv.data(), A.kv.data() + d, 2 * (size_t)d, A.o.data(), B, Tt, Ts, H, d / H, 0);
  std::vector<S> proj((size_t)N * d);
  linear_fwd<S>(A.o.data(), P + tab[e + 6].offset, P + tab[e + 7].offset, proj.data(), N, d, d);
  for (size_t i = 0; i < y.size(); ++i) y[i] += proj[i];
}

// dmem receives (+=) the gradient that reaches the encoder output through this sub-block.
template <class S>
void cross_block_bwd(const S* P, S* G, const std::vector<ParamEntry>& tab, size_t e, const CrossActs<S>& A,
                     const std::vector<S>& mem, std::vector<S>& dy, std::vector<S>& dmem, int B, int Tt, int Ts, int d,
                     int H) {
  const int N = B * Tt, Ns = B * Ts;
  std::vector<S> dO((size_t)N * d);
  linear_bwd<S>(A.o.data(), P + tab[e + 6].offset, dy.data(), dO.data(), G + tab[e + 6].offset, G + tab[e + 7].offset, N, d, d);
  std::vector<S> dq((size_t)N * d), dkv((size_t)Ns * 2 * d);
  mha_bwd<S>(A.q.data(), (size_t)d, A.kv.data(), A.kv.data() + d, 2 * (size_t)d, dO.data(), dq.data(), (size_t)d,
             dkv.data(), dkv.data() + d, 2 * (size_t)d, B, Tt, Ts, H, d / H, 0);
  std::vector<S> dm((size_t)Ns * d);
  linear_bwd<S>(mem.data(), P + tab[e + 4].offset, dkv.data(), dm.data(), G + tab[e + 4].offset, G + tab[e + 5].offset, Ns, d, 2 * d);
  for (size_t i = 0; i < dmem.size(); ++i) dmem[i] += dm[i];
  std::vector<S> da((size_t)N * d);
  linear_bwd<S>(A.a.data(), P + tab[e + 2].offset, dq.data(), da.data(), G + tab[e + 2].offset, G + tab[e + 3].offset, N, d, d);
  std::vector<S> dxl((size_t)N * d);
  layernorm_bwd<S>(da.data(), A.x_in.data(), P + tab[e].offset, dxl.data(), G + tab[e].offset, G + tab[e + 1].offset, N, d);
  for (size_t i = 0; i < dy.size(); ++i) dy[i] += dxl[i];
}

// x += gelu(LN(x) W1 + b1) W2 + b2; params at tab[e .. e+5].
template <class S>
void ffn_block_fwd(const S* P, const std::vector<ParamEntry>& tab, size_t e, std::vector<S>& x, FfnActs<S>& A, int N,
                   int d, int F) {
  A.x_in = x;
  A.m.resize((size_t)N * d);
  layernorm_fwd<S>(x.data(), P + tab[e].offset, P + tab[e + 1].offset, A.m.data(), nullptr, nullptr, N, d);
  A.u.resize((size_t)N * F);
  linear_fwd<S>(A.m.data(), P + tab[e + 2].offset, P + tab[e + 3].offset, A.u.data(), N, d, F);
  A.h.resize((size_t)N * F);
  for (size_t i = 0; i < A.u.size(); ++i) A.h[i] = gelu<S>(A.u[i]);
  std::vector<S> proj((size_t)N * d);
  linear_fwd<S>(A.h.data(), P + tab[e + 4].offset, P + tab[e + 5].offset, proj.data(), N, F, d);
  for (size_t i = 0; i < x.size(); ++i) x[i] += proj[i];
}

template <class S>
void ffn_block_bwd(const S* P, S* G, const std::vector<ParamEntry>& tab, size_t e, const FfnActs<S>& A,
                   std::vector<S>& dx, int N, int d, int F) {
  std::vector<S> dh((size_t)N * F);
  linear_bwd<S>(A.h.data(), P + tab[e + 4].offset, dx.data(), dh.data(), G + tab[e + 4].offset, G + tab[e + 5].offset, N, F, d);
  std::vector<S> du((size_t)N * F);
  for (size_t i = 0; i < du.size(); ++i) du[i] = dh[i] * gelu_grad<S>(A.u[i]);
  std::vector<S> dm((size_t)N * d);
  linear_bwd<S>(A.m.data(), P + tab[e + 2].offset, du.data(), dm.data(), G + tab[e + 2].offset, G + tab[e + 3].offset, N, d, F);
  std::vector<S> dxl((size_t)N * d);
  layernorm_bwd<S>(dm.data(), A.x_in.data(), P + tab[e].offset, dxl.data(), G + tab[e].offset, G + tab[e + 1].offset, N, d);
  for (size_t i = 0; i < dx.size(); ++i) dx[i] += dxl[i];
}

// One full train step (E1, E2).  src [B, Ts], tgt [B, Tt+1].  P is updated in place when opt.kind != 0;
// G receives the gradients (every parameter is used exactly once, so each entry is written once);
// logits (optional) [B*Tt, V]; do_bwd = 0 stops after the loss.
template <class S>
void encdec_train_step(const EncDecShape& s, S* P, S* M, S* Vv, const int32_t* src, const int32_t* tgt_tokens,
                       const OptConfig& opt, S* loss, S* G, S* logits, int do_bwd) {
  const int d = s.d, V = s.V, Ns = s.B * s.Ts, Nt = s.B * s.Tt;
  const auto tab = encdec_param_table(s);
  const size_t total = encdec_param_total(s);
  const size_t enc0 = 2, enc_tail = enc0 + (size_t)s.Le * kEncLayerParams;
  const size_t dec_emb = enc_tail + 2, dec0 = dec_emb + 2, dec_tail = dec0 + (size_t)s.Ld * kDecLayerParams;
  std::vector<int32_t> inp(Nt), tgt(Nt);
  for (int b = 0; b < s.B; ++b)
    for (int t = 0; t < s.Tt; ++t) {
      inp[b * s.Tt + t] = tgt_tokens[b * (s.Tt + 1) + t];
      tgt[b * s.Tt + t] = tgt_tokens[b * (s.Tt + 1) + t + 1];
    }

  // encoder
  std::vector<S> x((size_t)Ns * d);
  embedding_fwd<S>(src, P + tab[0].offset, P + tab[1].offset, x.data(), s.B, s.Ts, d);
  std::vector<SelfActs<S>> enc_self(s.Le);
  std::vector<FfnActs<S>> enc_ffn(s.Le);
  for (int l = 0; l < s.Le; ++l) {
    const size_t e = enc0 + (size_t)l * kEncLayerParams;
    self_block_fwd<S>(P, tab, e, x, enc_self[l], s.B, s.Ts, d, s.H, 0);
    ffn_block_fwd<S>(P, tab, e + 6, x, enc_ffn[l], Ns, d, s.F);
  }
  std::vector<S> mem((size_t)Ns * d);
  layernorm_fwd<S>(x.data(), P + tab[enc_tail].offset, P + tab[enc_tail + 1].offset, mem.data(), nullptr, nullptr, Ns, d);

  // decoder
  std::vector<S> y((size_t)Nt * d);
  embedding_fwd<S>(inp.data(), P + tab[dec_emb].offset, P + tab[dec_emb + 1].offset, y.data(), s.B, s.Tt, d);
  std::vector<SelfActs<S>> dec_self(s.Ld);
  std::vector<CrossActs<S>> dec_cross(s.Ld);
  std::vector<FfnActs<S>> dec_ffn(s.Ld);
  for (int l = 0; l < s.Ld; ++l) {
    const size_t e = dec0 + (size_t)l * kDecLayerParams;
    self_block_fwd<S>(P, tab, e, y, dec_self[l], s.B, s.Tt, d, s.H, 1);
    cross_block_fwd<S>(P, tab, e + 6, y, mem, dec_cross[l], s.B, s.Tt, s.Ts, d, s.H);
    ffn_block_fwd<S>(P, tab, e + 14, y, dec_ffn[l], Nt, d, s.F);
  }
  std::vector<S> yf((size_t)Nt * d), z((size_t)Nt * V);
  layernorm_fwd<S>(y.data(), P + tab[dec_tail].offset, P + tab[dec_tail + 1].offset, yf.data(), nullptr, nullptr, Nt, d);
  linear_fwd<S>(yf.data(), P + tab[dec_tail + 2].offset, nullptr, z.data(), Nt, d, V);
  if (logits) std::memcpy(logits, z.data(), z.size() * sizeof(S));
  std::vector<S> dz(do_bwd ? z.size() : 0);
  softmax_xent<S>(z.data(), tgt.data(), Nt, V, loss, do_bwd ? dz.data() : nullptr);
  if (!do_bwd) return;

  std::fill(G, G + total, S(0));
  std::vector<S> dyf((size_t)Nt * d), dy((size_t)Nt * d);
  linear_bwd<S>(yf.data(), P + tab[dec_tail + 2].offset, dz.data(), dyf.data(), G + tab[dec_tail + 2].offset, nullptr, Nt, d, V);
  layernorm_bwd<S>(dyf.data(), y.data(), P + tab[dec_tail].offset, dy.data(), G + tab[dec_tail].offset, G + tab[dec_tail + 1].offset, Nt, d);
  std::vector<S> dmem((size_t)Ns * d, S(0));
  for (int l = s.Ld - 1; l >= 0; --l) {
    const size_t e = dec0 + (size_t)l * kDecLayerParams;
    ffn_block_bwd<S>(P, G, tab, e + 14, dec_ffn[l], dy, Nt, d, s.F);
    cross_block_bwd<S>(P, G, tab, e + 6, dec_cross[l], mem, dy, dmem, s.B, s.Tt, s.Ts, d, s.H);
    self_block_bwd<S>(P, G, tab, e, dec_self[l], dy, s.B, s.Tt, d, s.H, 1);
  }
  embedding_bwd<S>(inp.data(), dy.data(), G + tab[dec_emb].offset, G + tab[dec_emb + 1].offset, s.B, s.Tt, d, V);

  std::vector<S> dx((size_t)Ns * d);
  layernorm_bwd<S>(dmem.data(), x.data(), P + tab[enc_tail].offset, dx.data(), G + tab[enc_tail].offset, G + tab[enc_tail + 1].offset, Ns, d);
  for (int l = s.Le - 1; l >= 0; --l) {
    const size_t e = enc0 + (size_t)l * kEncLayerParams;
    ffn_block_bwd<S>(P, G, tab, e + 6, enc_ffn[l], dx, Ns, d, s.F);
    self_block_bwd<S>(P, G, tab, e, enc_self[l], dx, s.B, s.Ts, d, s.H, 0);
  }
  embedding_bwd<S>(src, dx.data(), G + tab[0].offset, G + tab[1].offset, s.B, s.Ts, d, V);

  if (opt.kind == 1) sgd<S>(P, G, total, S(opt.lr));
  if (opt.kind == 2) adam<S>(P, M, Vv, G, total, S(opt.lr), S(opt.beta1), S(opt.beta2), S(opt.eps), opt.t);
}

}  // namespace oracle
