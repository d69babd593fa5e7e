// Choice of kernel per op and compute dtype: MFMA kernels for bf16 where they apply, plain kernels
// for fp32 and for shapes the MFMA kernels do not take.
#include <stdlib.h>
#include "common.h"

namespace lp {

hipError_t attn_fwd_plain(const OpCtx& c, const void* qkv, void* o, float* lse, int B, int S, int H, int dh, int causal);
hipError_t attn_bwd_plain(const OpCtx& c, const void* qkv, const void* o, const float* lse, const void* dout,
                          void* dqkv, float* delta, int B, int S, int H, int dh, int causal);
hipError_t conv_fwd_plain(const OpCtx& c, const ConvArgs& a, const void* x, const void* w, void* out);
hipError_t conv_bwd_data_plain(const OpCtx& c, const ConvArgs& a, const void* dout, const void* w, void* dx,
                               const void* add = nullptr);
hipError_t conv_bwd_weight_plain(const OpCtx& c, const ConvArgs& a, const void* dout, const void* x, float* dw,
                                 int accumulate);

hipError_t attn_fwd_mfma(const OpCtx& c, const void* qkv, void* o, float* lse, int B, int S, int H, int causal);
hipError_t attn_bwd_mfma(const OpCtx& c, const void* qkv, const void* o, const float* lse, const void* dout,
                         void* dqkv, float* delta, int B, int S, int H, int causal);

bool conv_mfma_ok(const OpCtx& c, const ConvArgs& a, const void* p0, const void* p1, const void* p2);
hipError_t conv_fwd_mfma(const OpCtx& c, const ConvArgs& a, const void* x, const void* w, void* out, ConvStats* st);
hipError_t conv_bwd_data_mfma(const OpCtx& c, const ConvArgs& a, const void* dout, const void* w, void* dx,
                              const void* add);
hipError_t conv_bwd_weight_mfma(const OpCtx& c, const ConvArgs& a, const void* dout, const void* x, float* dw,
                                int accumulate);
static bool plain_conv() {
  static int v = -1;
  if (v < 0) { const char* s = getenv("LP_PLAIN_CONV"); v = (s && s[0] == '1') ? 1 : 0; }
  return v != 0;
}

static bool use_mfma_attn(const OpCtx& c, int dh) {
  static int plain = -1;
  if (plain < 0) { const char* s = getenv("LP_PLAIN_ATTN"); plain = (s && s[0] == '1') ? 1 : 0; }
  return c.dt == BF16 && dh == 64 && !plain;
}

hipError_t op_attn_fwd(const OpCtx& c, const void* qkv, void* o, float* lse, int B, int S, int H, int dh, int causal) {
  ProfScope prof_(c, KC_ATTN_FWD);
  if (use_mfma_attn(c, dh)) return attn_fwd_mfma(c, qkv, o, lse, B, S, H, causal);
  return attn_fwd_plain(c, qkv, o, lse, B, S, H, dh, causal);
}
hipError_t op_attn_bwd(const OpCtx& c, const void* qkv, const void* o, const float* lse, const void* dout, void* dqkv,
                       float* delta, int B, int S, int H, int dh, int causal) {
  ProfScope prof_(c, KC_ATTN_BWD);
  if (use_mfma_attn(c, dh)) return attn_bwd_mfma(c, qkv, o, lse, dout, dqkv, delta, B, S, H, causal);
  return attn_bwd_plain(c, qkv, o, lse, dout, dqkv, delta, B, S, H, dh, causal);
}
hipError_t op_conv_fwd(const OpCtx& c, const ConvArgs& a, const void* x, const void* w, void* out, ConvStats* stats) {
  ProfScope prof_(c, KC_CONV, 2.0 * a.N * a.P * a.Q * a.O * a.R * a.S * a.C);
  if (stats) { stats->nslab = 0; stats->slab_rows = 0; }
  if (!plain_conv() && conv_mfma_ok(c, a, x, w, out)) return conv_fwd_mfma(c, a, x, w, out, stats);
  return conv_fwd_plain(c, a, x, w, out);
}
hipError_t op_conv_bwd_data(const OpCtx& c, const ConvArgs& a, const void* dout, const void* w, void* dx,
                            const void* add) {
  ProfScope prof_(c, KC_CONV, 2.0 * a.N * a.P * a.Q * a.O * a.R * a.S * a.C);
  if (!plain_conv() && conv_mfma_ok(c, a, dout, w, dx) && (!add || ((uintptr_t)add & 15) == 0))
    return conv_bwd_data_mfma(c, a, dout, w, dx, add);
  return conv_bwd_data_plain(c, a, dout, w, dx, add);
}
hipError_t op_conv_bwd_weight(const OpCtx& c, const ConvArgs& a, const void* dout, const void* x, float* dw,
                              int accumulate) {
  ProfScope prof_(c, KC_CONV, 2.0 * a.N * a.P * a.Q * a.O * a.R * a.S * a.C);
  if (!plain_conv() && conv_mfma_ok(c, a, dout, x, dw)) return conv_bwd_weight_mfma(c, a, dout, x, dw, accumulate);
  return conv_bwd_weight_plain(c, a, dout, x, dw, accumulate);
}

}  // namespace lp
