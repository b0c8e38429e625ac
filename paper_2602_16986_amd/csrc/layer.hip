// C-ABI entry points of one whole HSTU layer (paper Eq. 1-5) with the selective activation rematerialisation of
// Section 4.2.2 and the layer pseudocode of the appendix: the forward keeps only the gate U, the attention output A and
// the statistics of the input norm; the backward rebuilds the normalised input, the U/V/Q/K projection and the gated
// norm output from them.  Declarations and argument meaning: include/hstu_attn.h.
#include "../../include/hstu_attn.h"
#include "hstu_common.h"
#include "hstu_kernels.h"
#include "profile.h"

using namespace hstu;

namespace {

constexpr size_t kAlign = 256;
constexpr size_t kGemmWorkspace = (size_t)64 << 20;     // scratch offered to the GEMM library (split-K partial sums)
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct LayerLayout {
  size_t attn, gemm, norm_partial, xn, pre, act, y, dy, dattn, dact, dxn, qscale, tn_partial, total;
  size_t attn_bytes;
};

hstu_attn_params attn_problem(const hstu_layer_params* p) {
  hstu_attn_params a = p->attn;
  const int64_t hd = (int64_t)a.num_heads * a.head_dim;
  a.row_stride_q = a.row_stride_k = a.row_stride_v = 4 * hd;     // column blocks of the fused projection buffer
  a.row_stride_o = hd;
  return a;
}

int validate_layer(const hstu_layer_params* p) {
  if (!p) return HSTU_ERR_NULL;
  if (p->attn.dtype != HSTU_BF16) return HSTU_ERR_UNSUPPORTED;
  if (p->embed_dim < 8 || p->embed_dim % 8 != 0 || p->embed_dim > 8192) return HSTU_ERR_UNSUPPORTED;
  if (p->attn.num_heads < 1 || p->attn.head_dim < 1) return HSTU_ERR_SHAPE;
  const int64_t hd = (int64_t)p->attn.num_heads * p->attn.head_dim;
  if (hd > 8192) return HSTU_ERR_UNSUPPORTED;
  if (p->attn.total_tokens < 0) return HSTU_ERR_SHAPE;
  if (p->attn.query_tail != 0) return HSTU_ERR_UNSUPPORTED;     // every step of the layer runs on all rows
  const int nq = (p->w1_q != nullptr) + (p->w1_scale != nullptr) + (p->w2_q != nullptr) + (p->w2_scale != nullptr);
  if (nq != 0 && nq != 4) return HSTU_ERR_NULL;
  if (nq == 4 && (!fp8_gemm_supported((int)(4 * hd), p->embed_dim) || !fp8_gemm_supported(p->embed_dim, (int)hd)))
    return HSTU_ERR_UNSUPPORTED;
  return HSTU_OK;
}

LayerLayout make_layer_layout(const hstu_layer_params* p, int for_backward) {
  LayerLayout l = {};
  const hstu_attn_params a = attn_problem(p);
  const size_t T = (size_t)a.total_tokens, E = (size_t)p->embed_dim, HD = (size_t)a.num_heads * a.head_dim;
  size_t off = 0;
  l.attn = off; l.attn_bytes = hstu_attn_workspace_bytes(&a, for_backward); off += align_up(l.attn_bytes);
  l.gemm = off; off += kGemmWorkspace;
  l.xn = off; off += align_up(T * E * 2);
  l.act = off; off += align_up(T * 4 * HD * 2);
  l.y = off; off += align_up(T * HD * 2);
  l.qscale = off; off += align_up(2 * T * sizeof(float));     // row scales of the FP8 forward (X, then Y)
  if (for_backward) {
    const size_t pe = hstu_gated_norm_bwd_workspace_bytes((int64_t)T, (int32_t)E);
    const size_t ph = hstu_gated_norm_bwd_workspace_bytes((int64_t)T, (int32_t)HD);
    l.norm_partial = off; off += align_up(pe > ph ? pe : ph);
    l.pre = off; off += align_up(T * 4 * HD * 2);
    l.dy = off; off += align_up(T * HD * 2);
    l.dattn = off; off += align_up(T * HD * 2);
    l.dact = off; off += align_up(T * 4 * HD * 2);
    l.dxn = off; off += align_up(T * E * 2);
    size_t tn = 0;                                     // partial tiles of the two weight-gradient products
    if (gemm_tn_supported((int)E, (int)HD)) tn = gemm_tn_workspace_bytes((int64_t)T, (int)E, (int)HD);
    if (gemm_tn_supported((int)(4 * HD), (int)E)) {
      const size_t t1 = gemm_tn_workspace_bytes((int64_t)T, (int)(4 * HD), (int)E);
      tn = t1 > tn ? t1 : tn;
    }
    l.tn_partial = off; off += align_up(tn);
  }
  l.total = off;
  return l;
}

inline bool bad16(const void* ptr) { return ((uintptr_t)ptr & 15u) != 0; }
inline int gemm_status(int rc) { return rc == 0 ? HSTU_OK : (rc == -2 ? HSTU_ERR_UNSUPPORTED : HSTU_ERR_LAUNCH); }

}  // namespace

extern "C" {

size_t hstu_layer_workspace_bytes(const hstu_layer_params* p, int for_backward) {
  if (validate_layer(p) != HSTU_OK) return 0;
  const hstu_attn_params a = attn_problem(p);
  if (hstu_attn_workspace_bytes(&a, for_backward) == 0) return 0;
  return make_layer_layout(p, for_backward).total;
}

int hstu_layer_fwd(const hstu_layer_params* p, const void* z, void* out, void* u_saved, void* attn_saved, float* mean,
                   float* rstd, void* workspace, size_t workspace_bytes, void* stream_) {
  int st = validate_layer(p);
  if (st != HSTU_OK) return st;
  hipStream_t stream = (hipStream_t)stream_;
  const hstu_attn_params ap = attn_problem(p);
  const int64_t T = ap.total_tokens, E = p->embed_dim, HD = (int64_t)ap.num_heads * ap.head_dim;
  if (T == 0 || ap.batch == 0) return HSTU_OK;
  if (!z || !out || !u_saved || !attn_saved || !mean || !rstd || !p->norm_w || !p->w1 || !p->gated_norm_w || !p->w2)
    return HSTU_ERR_NULL;
  if (bad16(z) || bad16(out) || bad16(u_saved) || bad16(attn_saved) || bad16(p->w1) || bad16(p->w2) || bad16(p->norm_w) ||
      bad16(p->gated_norm_w) || bad16(p->w1_q) || bad16(p->w1_scale) || bad16(p->w2_q) || bad16(p->w2_scale))
    return HSTU_ERR_SHAPE;
  const LayerLayout l = make_layer_layout(p, 0);
  if (l.attn_bytes == 0) return HSTU_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < l.total) return HSTU_ERR_WORKSPACE;
  unsigned char* ws = (unsigned char*)workspace;
  __bf16* xn = (__bf16*)(ws + l.xn);
  __bf16* act = (__bf16*)(ws + l.act);
  __bf16* y = (__bf16*)(ws + l.y);
  const bool fp8 = p->w1_q != nullptr;
  float* xscale = (float*)(ws + l.qscale);
  float* yscale = xscale + T;
  if (fp8) {  // Eq. 1 with the row-wise quantisation fused in: X leaves the norm kernel as E4M3 codes (in the X buffer) and scales
    ProfScope ps("layer_norm_quant", stream);
    NormFwdArgs n = {};
    n.T = T; n.D = (int32_t)E; n.dtype = HSTU_BF16; n.a = z; n.sa = E; n.u = nullptr; n.su = 0; n.gamma = p->norm_w; n.beta = nullptr;
    n.eps = p->norm_eps; n.y = nullptr; n.sy = E; n.mean = mean; n.rstd = rstd; n.stats_in = 0;
    if (launch_norm_quant_fwd(n, xn, E, xscale, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
  } else {  // Eq. 1: X = LayerNorm(Z) * norm_w; the statistics are kept for the backward
    ProfScope ps("layer_norm_fwd", stream);
    NormFwdArgs n = {};
    n.T = T; n.D = (int32_t)E; n.dtype = HSTU_BF16; n.a = z; n.sa = E; n.u = nullptr; n.su = 0; n.gamma = p->norm_w; n.beta = nullptr;
    n.eps = p->norm_eps; n.y = xn; n.sy = E; n.mean = mean; n.rstd = rstd; n.stats_in = 0;
    if (launch_norm_fwd(n, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
  }
  if (fp8) {  // Eq. 2 on the quantised operands, SiLU in the GEMM's epilogue, the gate written straight to the saved tensor
    ProfScope ps("fp8_gemm_uvqk", stream);
    if (launch_fp8_gemm_silu(T, (int)(4 * HD), (int)E, xn, xscale, p->w1_q, p->w1_scale, act, u_saved, (int)HD, stream) != hipSuccess)
      return HSTU_ERR_LAUNCH;
  } else {
    // Eq. 2: [U V Q K] = SiLU(X W1^T), SiLU in the GEMM library's epilogue: the gate's rows of W1 go straight to the saved-U
    // tensor, the V, Q, K rows to their column blocks of the projection buffer.  A library build without such a kernel
    // (-2) gets the plain product and a SiLU pass.
    bool fused;
    {
      ProfScope ps("gemm_uvqk", stream);
      int rc = gemm_bf16(kGemmNT, T, HD, E, xn, E, p->w1, E, nullptr, 0, u_saved, HD, false, ws + l.gemm, kGemmWorkspace, stream, true);
      if (rc == 0)
        rc = gemm_bf16(kGemmNT, T, 3 * HD, E, xn, E, (const __bf16*)p->w1 + HD * E, E, nullptr, 0, act + HD, 4 * HD, false, ws + l.gemm,
                       kGemmWorkspace, stream, true);
      fused = rc == 0;
      if (rc == -2) rc = gemm_bf16(kGemmNT, T, 4 * HD, E, xn, E, p->w1, E, nullptr, 0, act, 4 * HD, false, ws + l.gemm, kGemmWorkspace, stream);
      if (rc != 0) return gemm_status(rc);
    }
    if (!fused) {
      ProfScope ps("silu_fwd", stream);
      if (launch_silu_fwd(T, (int)(4 * HD), act, act, u_saved, (int)HD, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
    }
  }
  // Eq. 3: A = attention(Q, K, V) on column blocks of the projection buffer
  st = hstu_attn_fwd(&ap, act + 2 * HD, act + 3 * HD, act + HD, attn_saved, ws + l.attn, l.attn_bytes, stream_);
  if (st != HSTU_OK) return st;
  if (fp8) {
    {  // Eq. 4 before f2 with the quantisation fused in
      ProfScope ps("gated_norm_quant", stream);
      NormFwdArgs n = {};
      n.T = T; n.D = (int32_t)HD; n.dtype = HSTU_BF16; n.a = attn_saved; n.sa = HD; n.u = u_saved; n.su = HD; n.gamma = p->gated_norm_w;
      n.beta = nullptr; n.eps = p->gated_norm_eps; n.y = nullptr; n.sy = HD; n.mean = nullptr; n.rstd = nullptr; n.stats_in = 0;
      if (launch_norm_quant_fwd(n, y, HD, yscale, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
    }
    {  // f2 and the residual (Eq. 5) in one FP8 GEMM: Z is its two-dimensional additive operand
      ProfScope ps("fp8_gemm_out", stream);
      if (launch_fp8_gemm_bias2d(T, (int)E, (int)HD, y, yscale, p->w2_q, p->w2_scale, z, out, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
    }
    return HSTU_OK;
  }
  {  // Eq. 4 before f2: Y = LayerNorm(A) * gated_norm_w (.) U
    ProfScope ps("gated_norm_fwd", stream);
    if (launch_gated_norm_fwd(T, (int)HD, HSTU_BF16, attn_saved, u_saved, p->gated_norm_w, nullptr, p->gated_norm_eps, y, nullptr, nullptr,
                              stream) != hipSuccess)
      return HSTU_ERR_LAUNCH;
  }
  {  // f2 and the residual (Eq. 5): out = Y W2^T + Z, the residual as the GEMM's additive operand
    ProfScope ps("gemm_out", stream);
    st = gemm_status(gemm_bf16(kGemmNT, T, E, HD, y, HD, p->w2, HD, z, E, out, E, false, ws + l.gemm, kGemmWorkspace, stream));
    if (st != HSTU_OK) return st;
  }
  return HSTU_OK;
}

int hstu_layer_bwd(const hstu_layer_params* p, const void* z, const void* u_saved, const void* attn_saved, const float* mean,
                   const float* rstd, const void* dout, void* dz, float* d_norm_w, float* d_w1, float* d_gated_norm_w,
                   float* d_w2, void* workspace, size_t workspace_bytes, void* stream_) {
  int st = validate_layer(p);
  if (st != HSTU_OK) return st;
  hipStream_t stream = (hipStream_t)stream_;
  const hstu_attn_params ap = attn_problem(p);
  const int64_t T = ap.total_tokens, E = p->embed_dim, HD = (int64_t)ap.num_heads * ap.head_dim;
  if (!d_norm_w || !d_w1 || !d_gated_norm_w || !d_w2) return HSTU_ERR_NULL;
  if (T == 0 || ap.batch == 0) {                      // no token: every weight gradient is zero
    if (launch_fill_zero(d_norm_w, (size_t)E, stream) != hipSuccess || launch_fill_zero(d_w1, (size_t)(4 * HD * E), stream) != hipSuccess ||
        launch_fill_zero(d_gated_norm_w, (size_t)HD, stream) != hipSuccess || launch_fill_zero(d_w2, (size_t)(E * HD), stream) != hipSuccess)
      return HSTU_ERR_LAUNCH;
    if (ap.d_rab_table && ap.num_buckets > 0 &&
        launch_fill_zero(ap.d_rab_table, (size_t)ap.num_heads * ap.num_buckets, stream) != hipSuccess)
      return HSTU_ERR_LAUNCH;
    return HSTU_OK;
  }
  if (!z || !u_saved || !attn_saved || !mean || !rstd || !dout || !dz || !p->norm_w || !p->w1 || !p->gated_norm_w || !p->w2)
    return HSTU_ERR_NULL;
  if (bad16(z) || bad16(u_saved) || bad16(attn_saved) || bad16(dout) || bad16(dz) || bad16(p->w1) || bad16(p->w2) ||
      bad16(p->norm_w) || bad16(p->gated_norm_w) || bad16(p->w1_q) || bad16(p->w1_scale))
    return HSTU_ERR_SHAPE;
  const LayerLayout l = make_layer_layout(p, 1);
  if (l.attn_bytes == 0) return HSTU_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < l.total) return HSTU_ERR_WORKSPACE;
  unsigned char* ws = (unsigned char*)workspace;
  __bf16* xn = (__bf16*)(ws + l.xn);
  __bf16* pre = (__bf16*)(ws + l.pre);
  __bf16* act = (__bf16*)(ws + l.act);
  __bf16* y = (__bf16*)(ws + l.y);
  __bf16* dy = (__bf16*)(ws + l.dy);
  __bf16* dattn = (__bf16*)(ws + l.dattn);
  __bf16* dact = (__bf16*)(ws + l.dact);
  __bf16* dxn = (__bf16*)(ws + l.dxn);
  float* partial = (float*)(ws + l.norm_partial);
  void* gws = ws + l.gemm;
  const bool fp8 = p->w1_q != nullptr;
  // Ordered by what each step needs, not by the forward's order.
  // No kernel of its own for the SiLU backward: every producer of a projection gradient multiplies by SiLU' as it stores.
  {  // Eq. 5 / f2, out = Y W2^T + Z:  dY = dout W2
    ProfScope ps("gemm_dy", stream);
    st = gemm_status(gemm_bf16(kGemmNN, T, HD, E, dout, E, p->w2, HD, nullptr, 0, dy, HD, false, gws, kGemmWorkspace, stream));
    if (st != HSTU_OK) return st;
  }
  {  // Eq. 1 again: the normalised input from the saved statistics (in bf16: the weight gradient needs it in any case)
    ProfScope ps("layer_norm_fwd", stream);
    NormFwdArgs n = {};
    n.T = T; n.D = (int32_t)E; n.dtype = HSTU_BF16; n.a = z; n.sa = E; n.u = nullptr; n.su = 0; n.gamma = p->norm_w; n.beta = nullptr;
    n.eps = p->norm_eps; n.y = xn; n.sy = E; n.mean = const_cast<float*>(mean); n.rstd = const_cast<float*>(rstd); n.stats_in = 1;
    if (launch_norm_fwd(n, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
  }
  if (fp8) {
    // the forward ran its first projection in FP8: rematerialise U, V, Q, K the same way, so that the backward differentiates
    // at the activations the forward produced (codes and scales of X go to the dX buffer, which is free until the end)
    float* xscale = (float*)(ws + l.qscale);
    {
      ProfScope ps("layer_norm_quant", stream);
      NormFwdArgs n = {};
      n.T = T; n.D = (int32_t)E; n.dtype = HSTU_BF16; n.a = z; n.sa = E; n.u = nullptr; n.su = 0; n.gamma = p->norm_w; n.beta = nullptr;
      n.eps = p->norm_eps; n.y = nullptr; n.sy = E; n.mean = nullptr; n.rstd = nullptr; n.stats_in = 0;
      if (launch_norm_quant_fwd(n, dxn, E, xscale, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
    }
    ProfScope ps("fp8_gemm_uvqk", stream);
    if (launch_fp8_gemm_bias2d(T, (int)(4 * HD), (int)E, dxn, xscale, p->w1_q, p->w1_scale, nullptr, pre, stream) != hipSuccess)
      return HSTU_ERR_LAUNCH;
  } else {  // rematerialise U, V, Q, K; the pre-activations stay for the SiLU backward
    ProfScope ps("gemm_uvqk", stream);
    st = gemm_status(gemm_bf16(kGemmNT, T, 4 * HD, E, xn, E, p->w1, E, nullptr, 0, pre, 4 * HD, false, gws, kGemmWorkspace, stream));
    if (st != HSTU_OK) return st;
  }
  {  // Eq. 4 backward: dA, d gated_norm_w and, through U = SiLU(gate pre-activation), the gate block of the projection gradient;
     // the same pass rebuilds Y from the saved A and U
    ProfScope ps("gated_norm_bwd", stream);
    NormBwdArgs n = {};
    n.T = T; n.D = (int32_t)HD; n.dtype = HSTU_BF16; n.dy = dy; n.sdy = HD; n.a = attn_saved; n.sa = HD; n.u = u_saved; n.su = HD;
    n.gamma = p->gated_norm_w; n.beta = nullptr; n.eps = p->gated_norm_eps; n.da = dattn; n.sda = HD; n.du = dact; n.sdu = 4 * HD;
    n.du_pre = pre; n.sdu_pre = 4 * HD;
    n.y_out = y; n.sy_out = HD;                            // Eq. 4 again: Y, for dW2 = dout^T Y further down
    n.residual = nullptr; n.sres = 0; n.dgamma = d_gated_norm_w; n.dbeta = nullptr;
    if (launch_norm_bwd(n, partial, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
  }
  {
    ProfScope ps("silu_fwd", stream);
    // (V, Q, K only: the gate's activation is the saved tensor, nothing reads it from this buffer)
    if (launch_silu_fwd(T, (int)(4 * HD), pre, act, nullptr, 0, stream, (int)HD) != hipSuccess) return HSTU_ERR_LAUNCH;
  }
  // attention backward: the gradients of the V, Q, K pre-activations land in their column blocks (SiLU' applied on the way out)
  st = attn_bwd_through_silu(&ap, act + 2 * HD, act + 3 * HD, act + HD, pre + 2 * HD, pre + 3 * HD, pre + HD, 4 * HD, dattn,
                             dact + 2 * HD, dact + 3 * HD, dact + HD, ws + l.attn, l.attn_bytes, stream_);
  if (st != HSTU_OK) return st;
  {  // pre = X W1^T:  dX = dpre W1,  dW1 = dpre^T X
    ProfScope ps("gemm_dxn", stream);
    st = gemm_status(gemm_bf16(kGemmNN, T, E, 4 * HD, dact, 4 * HD, p->w1, E, nullptr, 0, dxn, E, false, gws, kGemmWorkspace, stream));
    if (st != HSTU_OK) return st;
  }
  {
    ProfScope ps("gemm_dw1", stream);
    if (gemm_tn_supported((int)(4 * HD), (int)E)) {
      if (launch_gemm_tn(T, (int)(4 * HD), (int)E, dact, 4 * HD, xn, E, d_w1, (float*)(ws + l.tn_partial), stream) != hipSuccess)
        return HSTU_ERR_LAUNCH;
    } else {
      st = gemm_status(gemm_bf16(kGemmTN, 4 * HD, E, T, dact, 4 * HD, xn, E, nullptr, 0, d_w1, E, true, gws, kGemmWorkspace, stream));
      if (st != HSTU_OK) return st;
    }
  }
  {  // weight gradients: this library's slab-split kernel when the widths are multiples of 128, else the GEMM library
    ProfScope ps("gemm_dw2", stream);
    if (gemm_tn_supported((int)E, (int)HD)) {
      if (launch_gemm_tn(T, (int)E, (int)HD, dout, E, y, HD, d_w2, (float*)(ws + l.tn_partial), stream) != hipSuccess) return HSTU_ERR_LAUNCH;
    } else {
      st = gemm_status(gemm_bf16(kGemmTN, E, HD, T, dout, E, y, HD, nullptr, 0, d_w2, HD, true, gws, kGemmWorkspace, stream));
      if (st != HSTU_OK) return st;
    }
  }
  {  // input norm backward; the residual's gradient (dout) is added in the same pass
    ProfScope ps("layer_norm_bwd", stream);
    NormBwdArgs n = {};
    n.T = T; n.D = (int32_t)E; n.dtype = HSTU_BF16; n.dy = dxn; n.sdy = E; n.a = z; n.sa = E; n.u = nullptr; n.su = 0;
    n.gamma = p->norm_w; n.beta = nullptr; n.eps = p->norm_eps; n.da = dz; n.sda = E; n.du = nullptr; n.sdu = 0;
    n.residual = dout; n.sres = E; n.dgamma = d_norm_w; n.dbeta = nullptr;
    if (launch_norm_bwd(n, partial, stream) != hipSuccess) return HSTU_ERR_LAUNCH;
  }
  return HSTU_OK;
}

int64_t hstu_layer_gemm_tunings(void) { return (int64_t)gemm_bf16_tunings(); }

}  // extern "C"
