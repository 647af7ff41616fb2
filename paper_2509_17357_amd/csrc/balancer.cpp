// Balancer split (Cronus appendix A, Algorithm 1, with the time models of section 4.4,
// Eq. 1-3): the partial prefill length that makes the partial prefill on the low-end
// instance and the remaining chunked prefill iterations on the high-end instance take
// about the same time.  Pure host arithmetic.
#include <cmath>
#include <cstdint>

#include "cronus.h"

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

struct Times {
  double prefill, chunked;
};

// The two modelled times for a partial prefill of l_p tokens.  Formulated around the
// remainder of the prompt: the chunked prefill instance gets L_c = L_in - L_p tokens in
// iterations of n_p; q whole iterations and r = L_c - q n_p left-over tokens mean
// q + (r > 0) iterations, and the prefill context that Algorithm 1 assigns to the last
// of them, L_p + q n_p, is L_in - r.  Twice the mean context of Eq. 1 with Eq. 3 is
// therefore the integer 2 L_in - r.  `decode_term` = k_ctxd * L_ctxd (Eq. 3's second term,
// the same for every candidate).  Every product and sum is rounded on its own (no fused
// multiply-add), left to right as Algorithm 1 prints the expression, so that the choice
// agrees with any other IEEE double evaluation of it.
Times model_times(const cronus_balancer_model& m, int64_t l_in, int64_t l_p, int64_t n_p, double decode_term) {
#pragma clang fp contract(off)
  Times t;
  t.prefill = m.k_p * (double)l_p + m.b_p;
  const int64_t rest = l_in - l_p;
  const int64_t whole = rest / n_p, left = rest - whole * n_p;
  const int64_t iterations = whole + (left != 0);
  const double per_iter = m.k_ctxp * (double)(2 * l_in - left) / 2.0 + decode_term + m.b_c;
  t.chunked = (double)iterations * per_iter;
  return t;
}

}  // namespace

extern "C" int cronus_balancer_split(const cronus_balancer_model* model, int64_t l_in, int64_t n_d,
                                     int64_t l_ctxd, int64_t n_free, int64_t* l_p, double* t_prefill,
                                     double* t_chunked) {
  constexpr int64_t kExact = (int64_t)1 << 52;  // integers below convert to double exactly
  if (!model || !l_p) return CRONUS_ERR_INVALID_ARG;
  if (model->block_size <= 0 || model->batch_tokens <= 0 || model->n_candidates <= 0) return CRONUS_ERR_INVALID_ARG;
  if (l_in <= 0 || n_d < 0 || n_d >= model->batch_tokens || l_ctxd < 0 || n_free < 0) return CRONUS_ERR_INVALID_ARG;
  if (l_in >= kExact / model->n_candidates || l_ctxd >= kExact) return CRONUS_ERR_INVALID_ARG;
  const int64_t n_p = model->batch_tokens - n_d;
  double decode_term;
  {
#pragma clang fp contract(off)
    decode_term = model->k_ctxd * (double)l_ctxd;
  }

  int64_t best = l_in;
  if (n_free >= ceil_div(l_in, model->block_size)) {
    double best_gap = INFINITY;
    for (int64_t j = 1; j <= model->n_candidates; ++j) {
      const int64_t cand = ceil_div(j * l_in, model->n_candidates);
      const Times t = model_times(*model, l_in, cand, n_p, decode_term);
      const double gap = std::fabs(t.prefill - t.chunked);
      if (j == 1 || gap < best_gap) {  // strict: the first of equal minima stays
        best = cand;
        best_gap = gap;
      }
    }
  }
  *l_p = best;
  if (t_prefill || t_chunked) {
    const Times t = model_times(*model, l_in, best, n_p, decode_term);
    if (t_prefill) *t_prefill = t.prefill;
    if (t_chunked) *t_chunked = t.chunked;
  }
  return CRONUS_OK;
}
