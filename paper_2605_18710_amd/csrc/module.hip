// Module step: the sequence of kernels that makes one forward and one backward pass of a
// module (Sec. 3.1: the unit that holds a quota), its parameter layout and its workspace.
// Everything is enqueued on the module's stream; nothing here synchronises the host.
#include <string.h>
#include <math.h>
#include <string>
#include <vector>
#include <new>
#include <algorithm>
#include "kernels.h"

struct mosaic_stream;
hipStream_t mosaic_stream_hip(const mosaic_stream* s);   // launcher.hip
int mosaic_stream_quota_or(const mosaic_stream* s, int fallback);

namespace {

struct TensorInfo {
  std::string name;
  int64_t offset, rows, cols;
};

struct LayerParams {           // element offsets into params / grads
  int64_t n1_g = -1, n1_b = -1, w_qkv = -1, b_qkv = -1, w_o = -1, b_o = -1;
  int64_t n2_g = -1, n2_b = -1, w_1 = -1, b_1 = -1, w_2 = -1, b_2 = -1;
};

struct LayerSaved {            // byte offsets into the workspace
  size_t u1, qkv, o, lse, st1, x1, st2, u2, z, a, y;
};

}  // namespace

struct mosaic_module {
  mosaic_module_desc d;
  size_t esize;
  int64_t T;
  std::vector<TensorInfo> tensors;
  std::vector<LayerParams> lp;
  std::vector<LayerSaved> ls;
  int64_t param_elems = 0;
  size_t ws_bytes = 0;
  // scratch byte offsets
  size_t s_dA, s_dZ, s_dU, s_dX1, s_dO, s_dQKV, s_delta, s_g0, s_g1, s_norm, s_colsum, s_mse, s_dyloss, s_splitk;
  size_t s_patches;
  size_t s_rope = 0;     // (cos, sin) table of the rotary embedding, when on
  size_t c_p1 = 0, c_z1 = 0, c_a1 = 0, c_p2 = 0, c_z2 = 0, c_dz2 = 0, c_dp2 = 0, c_da1 = 0, c_dz1 = 0, c_dp1 = 0;   // conv stem
  // bound buffers
  char* params = nullptr;
  char* grads = nullptr;
  char* ws = nullptr;
  const int32_t* ids = nullptr;
  const int32_t* img_counts = nullptr;   // TEXT_STEM: per-sample image-token counts, optional
  const void* last_x = nullptr;
  bool forward_done = false;
};

namespace {

int64_t add_tensor(mosaic_module* m, const std::string& name, int64_t rows, int64_t cols) {
  const int64_t off = m->param_elems;
  m->tensors.push_back({name, off, rows, cols});
  int64_t n = rows * cols;
  n = (n + 7) / 8 * 8;          // keep every tensor 16-byte aligned in both dtypes
  m->param_elems += n;
  return off;
}

size_t take(size_t* cur, size_t bytes) {
  const size_t off = *cur;
  *cur = align_up(off + bytes, 256);
  return off;
}

mosaic_status validate(const mosaic_module_desc& d) {
  if (d.dtype != MOSAIC_F32 && d.dtype != MOSAIC_BF16) MOSAIC_FAIL(MOSAIC_EINVAL, "bad dtype %d", d.dtype);
  if (d.batch <= 0 || d.seq <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "batch and seq must be positive");
  const int vn = d.dtype == MOSAIC_BF16 ? 8 : 4;
  switch (d.kind) {
    case MOSAIC_ENCODER:
    case MOSAIC_DECODER:
      if (d.layers <= 0 || d.hidden <= 0 || d.heads <= 0 || d.mlp <= 0)
        MOSAIC_FAIL(MOSAIC_EINVAL, "layers, hidden, heads and mlp must be positive");
      if (d.hidden % d.heads) MOSAIC_FAIL(MOSAIC_EINVAL, "hidden %d is not a multiple of heads %d", d.hidden, d.heads);
      if (d.hidden / d.heads > 128) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "head size %d > 128", d.hidden / d.heads);
      if (d.hidden % vn || d.mlp % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "hidden and mlp must be multiples of %d", vn);
      if (d.norm != MOSAIC_LAYERNORM && d.norm != MOSAIC_RMSNORM) MOSAIC_FAIL(MOSAIC_EINVAL, "bad norm %d", d.norm);
      if (d.act != MOSAIC_GELU && d.act != MOSAIC_SWIGLU && d.act != MOSAIC_GELU_TANH) MOSAIC_FAIL(MOSAIC_EINVAL, "bad activation %d", d.act);
      if (d.kv_heads < 0 || (d.kv_heads > 0 && d.heads % d.kv_heads)) MOSAIC_FAIL(MOSAIC_EINVAL, "kv_heads %d must divide heads %d", d.kv_heads, d.heads);
      if (d.kv_heads > 0 && ((d.hidden / d.heads) * d.kv_heads) % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "key/value width must be a multiple of %d", vn);
      if (!(d.rope_base >= 0.f)) MOSAIC_FAIL(MOSAIC_EINVAL, "rope_base must be 0 (off) or positive");
      if (d.rope_base > 0.f && (d.hidden / d.heads) % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "rotary embedding needs a head size that is a multiple of %d", vn);
      if (!(d.eps > 0.f)) MOSAIC_FAIL(MOSAIC_EINVAL, "eps must be positive");
      break;
    case MOSAIC_PROJECTOR:
      if (d.in_dim <= 0 || d.out_dim <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "projector needs in_dim and out_dim");
      if (d.in_dim % vn || d.out_dim % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "projector widths must be multiples of %d", vn);
      break;
    case MOSAIC_PATCH_STEM: {
      if (d.in_dim <= 0 || d.hidden <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "stem needs in_dim and hidden");
      if (d.hidden % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "hidden must be a multiple of %d", vn);
      if (d.patch < 0) MOSAIC_FAIL(MOSAIC_EINVAL, "negative patch");
      if (d.patch > 0) {
        const int g = (int)lround(sqrt((double)d.seq));
        if (g * g != d.seq) MOSAIC_FAIL(MOSAIC_EINVAL, "seq %d is not a square patch grid", d.seq);
        if (d.in_dim != 3 * d.patch * d.patch) MOSAIC_FAIL(MOSAIC_EINVAL, "in_dim must be 3*patch*patch");
      }
      break;
    }
    case MOSAIC_CONV_STEM:
      if (d.in_dim <= 0 || d.hidden <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "conv stem needs in_dim and hidden");
      if (d.in_dim % vn || d.hidden % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "in_dim and hidden must be multiples of %d", vn);
      break;
    case MOSAIC_TEXT_STEM:
      if (d.hidden <= 0 || d.vocab <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "text stem needs hidden and vocab");
      if (d.n_img < 0 || d.n_img > d.seq) MOSAIC_FAIL(MOSAIC_EINVAL, "n_img must lie in [0, seq]");
      if (d.hidden % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "hidden must be a multiple of %d", vn);
      break;
    default:
      MOSAIC_FAIL(MOSAIC_EINVAL, "bad module kind %d", d.kind);
  }
  return MOSAIC_OK;
}

// width of a packed [q | k | v] row: heads query heads, kv key and value heads each
inline int64_t qkv_width(const mosaic_module_desc& d) {
  const int kv = d.kv_heads > 0 ? d.kv_heads : d.heads;
  return (int64_t)(d.heads + 2 * kv) * (d.hidden / d.heads);
}
inline int kv_heads_of(const mosaic_module_desc& d) { return d.kv_heads > 0 ? d.kv_heads : d.heads; }

void build_layout(mosaic_module* m) {
  const mosaic_module_desc& d = m->d;
  const int64_t T = m->T, h = d.hidden, f = d.mlp;
  const size_t es = m->esize;
  size_t cur = 0;
  if (d.kind == MOSAIC_ENCODER || d.kind == MOSAIC_DECODER) {
    const bool ln = d.norm == MOSAIC_LAYERNORM, glu = d.act == MOSAIC_SWIGLU;
    const int64_t qw = qkv_width(d);
    const char* nn = ln ? "ln" : "rms";
    for (int l = 0; l < d.layers; ++l) {
      const std::string p = "L" + std::to_string(l) + ".";
      LayerParams q;
      q.n1_g = add_tensor(m, p + nn + "1_g", 1, h);
      if (ln) q.n1_b = add_tensor(m, p + nn + "1_b", 1, h);
      q.w_qkv = add_tensor(m, p + "w_qkv", h, qw);
      if (d.bias) q.b_qkv = add_tensor(m, p + "b_qkv", 1, qw);
      q.w_o = add_tensor(m, p + "w_o", h, h);
      if (d.bias) q.b_o = add_tensor(m, p + "b_o", 1, h);
      q.n2_g = add_tensor(m, p + nn + "2_g", 1, h);
      if (ln) q.n2_b = add_tensor(m, p + nn + "2_b", 1, h);
      if (glu) {
        q.w_1 = add_tensor(m, p + "w_gu", h, 2 * f);
        if (d.bias) q.b_1 = add_tensor(m, p + "b_gu", 1, 2 * f);
        q.w_2 = add_tensor(m, p + "w_down", f, h);
        if (d.bias) q.b_2 = add_tensor(m, p + "b_down", 1, h);
      } else {
        q.w_1 = add_tensor(m, p + "w_1", h, f);
        if (d.bias) q.b_1 = add_tensor(m, p + "b_1", 1, f);
        q.w_2 = add_tensor(m, p + "w_2", f, h);
        if (d.bias) q.b_2 = add_tensor(m, p + "b_2", 1, h);
      }
      m->lp.push_back(q);
      LayerSaved s;
      const int64_t zf = glu ? 2 * f : f;
      s.u1 = take(&cur, T * h * es);
      s.qkv = take(&cur, T * qw * es);
      s.o = take(&cur, T * h * es);
      s.lse = take(&cur, (size_t)d.batch * d.heads * d.seq * sizeof(float));
      s.st1 = take(&cur, T * 2 * sizeof(float));
      s.x1 = take(&cur, T * h * es);
      s.st2 = take(&cur, T * 2 * sizeof(float));
      s.u2 = take(&cur, T * h * es);
      s.z = take(&cur, T * zf * es);
      s.a = take(&cur, T * f * es);
      s.y = (l + 1 < d.layers) ? take(&cur, T * h * es) : 0;
      m->ls.push_back(s);
    }
    const int64_t zf = glu ? 2 * f : f;
    m->s_dA = take(&cur, T * f * es);
    m->s_dZ = take(&cur, T * zf * es);
    m->s_dU = take(&cur, T * h * es);
    m->s_dX1 = take(&cur, T * h * es);
    m->s_dO = take(&cur, T * h * es);
    m->s_dQKV = take(&cur, T * qw * es);
    m->s_delta = take(&cur, (size_t)d.batch * d.heads * d.seq * sizeof(float));
    m->s_g0 = take(&cur, T * h * es);
    m->s_g1 = take(&cur, T * h * es);
    m->s_norm = take(&cur, norm_bwd_scratch_bytes(h));
    const int64_t widest = (qw > zf) ? qw : zf;
    m->s_colsum = take(&cur, colsum_scratch_bytes(widest));
    size_t sk = gemm_splitk_scratch_bytes(h, qw, T);
    sk = std::max(sk, gemm_splitk_scratch_bytes(h, h, T));
    sk = std::max(sk, gemm_splitk_scratch_bytes(h, zf, T));
    sk = std::max(sk, gemm_splitk_scratch_bytes(f, h, T));
    m->s_splitk = take(&cur, sk);
    if (d.rope_base > 0.f) m->s_rope = take(&cur, rope_table_bytes(d.seq, (int)(h / d.heads)));
  } else if (d.kind == MOSAIC_PROJECTOR) {
    LayerParams q;
    q.w_1 = add_tensor(m, "w_1", d.in_dim, d.out_dim);
    q.b_1 = add_tensor(m, "b_1", 1, d.out_dim);
    q.w_2 = add_tensor(m, "w_2", d.out_dim, d.out_dim);
    q.b_2 = add_tensor(m, "b_2", 1, d.out_dim);
    m->lp.push_back(q);
    LayerSaved s = {};
    s.z = take(&cur, T * d.out_dim * es);
    s.a = take(&cur, T * d.out_dim * es);
    m->ls.push_back(s);
    m->s_dA = take(&cur, T * d.out_dim * es);
    m->s_dZ = take(&cur, T * d.out_dim * es);
    m->s_colsum = take(&cur, colsum_scratch_bytes(d.out_dim));
    m->s_splitk = take(&cur, std::max(gemm_splitk_scratch_bytes(d.out_dim, d.out_dim, T),
                                      gemm_splitk_scratch_bytes(d.in_dim, d.out_dim, T)));
  } else if (d.kind == MOSAIC_PATCH_STEM) {
    LayerParams q;
    q.w_1 = add_tensor(m, "w_stem", d.in_dim, h);
    q.b_1 = add_tensor(m, "b_stem", 1, h);
    q.w_2 = add_tensor(m, "pos", d.seq, h);
    m->lp.push_back(q);
    m->s_patches = take(&cur, T * d.in_dim * es);
    m->s_colsum = take(&cur, colsum_scratch_bytes(h));
    m->s_splitk = take(&cur, gemm_splitk_scratch_bytes(d.in_dim, h, T));
  } else if (d.kind == MOSAIC_CONV_STEM) {
    LayerParams q;
    const int64_t C = d.in_dim, Tin = 2 * T;            // input frames = 2 * seq per sample
    q.w_1 = add_tensor(m, "w_c1", 3 * C, h);
    q.b_1 = add_tensor(m, "b_c1", 1, h);
    q.w_2 = add_tensor(m, "w_c2", 3 * h, h);
    q.b_2 = add_tensor(m, "b_c2", 1, h);
    q.w_o = add_tensor(m, "pos", d.seq, h);
    m->lp.push_back(q);
    m->c_p1 = take(&cur, Tin * 3 * C * es);
    m->c_z1 = take(&cur, Tin * h * es);
    m->c_a1 = take(&cur, Tin * h * es);
    m->c_p2 = take(&cur, T * 3 * h * es);
    m->c_z2 = take(&cur, T * h * es);
    m->c_dz2 = take(&cur, T * h * es);
    m->c_dp2 = take(&cur, T * 3 * h * es);
    m->c_da1 = take(&cur, Tin * h * es);
    m->c_dz1 = take(&cur, Tin * h * es);
    m->c_dp1 = take(&cur, Tin * 3 * C * es);
    m->s_colsum = take(&cur, colsum_scratch_bytes(h));
    m->s_splitk = take(&cur, std::max(gemm_splitk_scratch_bytes(3 * C, h, Tin), gemm_splitk_scratch_bytes(3 * h, h, T)));
  } else {  // TEXT_STEM
    LayerParams q;
    q.w_1 = add_tensor(m, "table", d.vocab, h);
    m->lp.push_back(q);
  }
  m->s_mse = take(&cur, mse_scratch_bytes());
  m->s_dyloss = take(&cur, mosaic_module_output_elems(m) * es);
  m->ws_bytes = cur;
}

inline void* P(const mosaic_module* m, int64_t off) { return off < 0 ? nullptr : m->params + off * m->esize; }
inline void* G(const mosaic_module* m, int64_t off) { return off < 0 ? nullptr : m->grads + off * m->esize; }
inline void* W(const mosaic_module* m, size_t off) { return m->ws + off; }

mosaic_status check_bound(const mosaic_module* m) {
  if (!m) MOSAIC_FAIL(MOSAIC_EINVAL, "null module");
  if (!m->params || !m->grads || !m->ws) MOSAIC_FAIL(MOSAIC_EINVAL, "module buffers are not bound");
  return MOSAIC_OK;
}

// ------------------------------------------------------------- transformer layers
mosaic_status layers_forward(mosaic_module* m, hipStream_t s, int q, const void* x, void* y) {
  const mosaic_module_desc& d = m->d;
  const int64_t T = m->T, h = d.hidden, f = d.mlp;
  const int dt = d.dtype;
  const bool glu = d.act == MOSAIC_SWIGLU;
  const void* xin = x;
  const bool rope = d.rope_base > 0.f;
  const int dh = (int)(h / d.heads), kvh = kv_heads_of(d);
  const int64_t qw = qkv_width(d);
  if (rope) MOSAIC_TRY(launch_rope_table(s, q, d.seq, dh, d.rope_base, W(m, m->s_rope)));
  for (int l = 0; l < d.layers; ++l) {
    const LayerParams& p = m->lp[l];
    const LayerSaved& sv = m->ls[l];
    void* yout = (l + 1 < d.layers) ? W(m, sv.y) : y;
    MOSAIC_TRY(launch_norm_fwd(s, q, dt, d.norm, T, h, d.eps, xin, P(m, p.n1_g), P(m, p.n1_b), W(m, sv.u1), (float*)W(m, sv.st1)));
    MOSAIC_TRY(launch_gemm(s, q, dt, true, false, T, qw, h, W(m, sv.u1), h, P(m, p.w_qkv), qw, W(m, sv.qkv), qw, P(m, p.b_qkv), nullptr));
    if (rope) MOSAIC_TRY(launch_rope(s, q, dt, d.batch, d.seq, d.heads, kvh, dh, +1, W(m, sv.qkv), W(m, m->s_rope)));   // saved rotated
    MOSAIC_TRY(launch_attention_fwd(s, q, dt, d.batch, d.seq, d.heads, kvh, dh, d.causal, W(m, sv.qkv), W(m, sv.o), (float*)W(m, sv.lse)));
    MOSAIC_TRY(launch_gemm(s, q, dt, true, false, T, h, h, W(m, sv.o), h, P(m, p.w_o), h, W(m, sv.x1), h, P(m, p.b_o), xin));
    MOSAIC_TRY(launch_norm_fwd(s, q, dt, d.norm, T, h, d.eps, W(m, sv.x1), P(m, p.n2_g), P(m, p.n2_b), W(m, sv.u2), (float*)W(m, sv.st2)));
    const int64_t zf = glu ? 2 * f : f;
    // up projection and activation in one launch where the matrix-core kernel takes it
    MOSAIC_TRY(launch_linear_act_fwd(s, q, dt, d.act, T, h, zf, W(m, sv.u2), P(m, p.w_1), P(m, p.b_1), W(m, sv.z), W(m, sv.a)));
    MOSAIC_TRY(launch_gemm(s, q, dt, true, false, T, h, f, W(m, sv.a), f, P(m, p.w_2), h, yout, h, P(m, p.b_2), W(m, sv.x1)));
    xin = yout;
  }
  return MOSAIC_OK;
}

mosaic_status layers_backward(mosaic_module* m, hipStream_t s, int q, const void* dy, void* dx) {
  const mosaic_module_desc& d = m->d;
  const int64_t T = m->T, h = d.hidden, f = d.mlp;
  const int dt = d.dtype;
  const bool glu = d.act == MOSAIC_SWIGLU;
  const int64_t zf = glu ? 2 * f : f;
  const int kvh = kv_heads_of(d);
  const int64_t qw = qkv_width(d);
  void* dA = W(m, m->s_dA); void* dZ = W(m, m->s_dZ); void* dU = W(m, m->s_dU);
  void* dX1 = W(m, m->s_dX1); void* dO = W(m, m->s_dO); void* dQKV = W(m, m->s_dQKV);
  void* nsc = W(m, m->s_norm); void* csc = W(m, m->s_colsum);
  const void* gin = dy;
  for (int l = d.layers - 1; l >= 0; --l) {
    const LayerParams& p = m->lp[l];
    const LayerSaved& sv = m->ls[l];
    const void* xin = (l == 0) ? m->last_x : W(m, m->ls[l - 1].y);
    void* gout = (l == 0) ? (dx ? dx : W(m, m->s_g0)) : W(m, (l & 1) ? m->s_g1 : m->s_g0);
    // MLP down projection
    MOSAIC_TRY(launch_gemm(s, q, dt, true, true, T, f, h, gin, h, P(m, p.w_2), h, dA, f, nullptr, nullptr));
    MOSAIC_TRY(launch_gemm(s, q, dt, false, false, f, h, T, W(m, sv.a), f, gin, h, G(m, p.w_2), h, nullptr, nullptr, W(m, m->s_splitk)));
    // Bias gradients are column sums of a layer's output gradient.  Each is formed by the kernel
    // that writes that gradient where there is one of ours: the first norm's backward of the
    // layer above (this layer's incoming gradient), the GELU backward, the second norm's
    // backward.  Only the top layer's incoming gradient and dQKV take a pass of their own.
    if (p.b_2 >= 0 && l == d.layers - 1) MOSAIC_TRY(launch_colsum(s, q, dt, T, h, gin, G(m, p.b_2), csc));
    // activation
    bool b1_done = false;
    if (glu) MOSAIC_TRY(launch_swiglu_bwd(s, q, dt, T, f, W(m, sv.z), dA, dZ));
    else if (d.act == MOSAIC_GELU_TANH) MOSAIC_TRY(launch_gelu_tanh_bwd(s, q, dt, T * f, W(m, sv.z), dA, dZ));
    else if (p.b_1 >= 0) { MOSAIC_TRY(launch_gelu_bwd_colsum(s, q, dt, T, f, W(m, sv.z), dA, dZ, G(m, p.b_1), csc)); b1_done = true; }
    else MOSAIC_TRY(launch_gelu_bwd(s, q, dt, T * f, W(m, sv.z), dA, dZ));
    // MLP up projection
    MOSAIC_TRY(launch_gemm(s, q, dt, false, false, h, zf, T, W(m, sv.u2), h, dZ, zf, G(m, p.w_1), zf, nullptr, nullptr, W(m, m->s_splitk)));
    if (p.b_1 >= 0 && !b1_done) MOSAIC_TRY(launch_colsum(s, q, dt, T, zf, dZ, G(m, p.b_1), csc));
    MOSAIC_TRY(launch_gemm(s, q, dt, true, true, T, h, zf, dZ, zf, P(m, p.w_1), zf, dU, h, nullptr, nullptr));
    // second norm; residual branch adds the incoming gradient
    MOSAIC_TRY(launch_norm_bwd(s, q, dt, d.norm, T, h, W(m, sv.x1), P(m, p.n2_g), (const float*)W(m, sv.st2), dU, gin, dX1, G(m, p.n2_g), G(m, p.n2_b), nsc,
                               G(m, p.b_o)));   // dX1 is the output gradient of the attention output projection
    // attention output projection
    MOSAIC_TRY(launch_gemm(s, q, dt, true, true, T, h, h, dX1, h, P(m, p.w_o), h, dO, h, nullptr, nullptr));
    MOSAIC_TRY(launch_gemm(s, q, dt, false, false, h, h, T, W(m, sv.o), h, dX1, h, G(m, p.w_o), h, nullptr, nullptr, W(m, m->s_splitk)));
    // attention
    MOSAIC_TRY(launch_attention_bwd(s, q, dt, d.batch, d.seq, d.heads, kvh, (int)(h / d.heads), d.causal, W(m, sv.qkv), W(m, sv.o),
                                    (const float*)W(m, sv.lse), dO, dQKV, (float*)W(m, m->s_delta)));
    // gradients of the rotated q, k go back through the transposed rotation (the table of
    // the forward pass is still in the workspace)
    if (d.rope_base > 0.f) MOSAIC_TRY(launch_rope(s, q, dt, d.batch, d.seq, d.heads, kvh, (int)(h / d.heads), -1, dQKV, W(m, m->s_rope)));
    // QKV projection
    MOSAIC_TRY(launch_gemm(s, q, dt, false, false, h, qw, T, W(m, sv.u1), h, dQKV, qw, G(m, p.w_qkv), qw, nullptr, nullptr, W(m, m->s_splitk)));
    if (p.b_qkv >= 0) MOSAIC_TRY(launch_colsum(s, q, dt, T, qw, dQKV, G(m, p.b_qkv), csc));
    MOSAIC_TRY(launch_gemm(s, q, dt, true, true, T, h, qw, dQKV, qw, P(m, p.w_qkv), qw, dU, h, nullptr, nullptr));
    // first norm
    MOSAIC_TRY(launch_norm_bwd(s, q, dt, d.norm, T, h, xin, P(m, p.n1_g), (const float*)W(m, sv.st1), dU, dX1, gout, G(m, p.n1_g), G(m, p.n1_b), nsc,
                               l > 0 ? G(m, m->lp[l - 1].b_2) : nullptr));   // gout is the incoming gradient of the layer below
    gin = gout;
  }
  return MOSAIC_OK;
}

// ---------------------------------------------------------------------- projector
mosaic_status projector_forward(mosaic_module* m, hipStream_t s, int q, const void* x, void* y) {
  const mosaic_module_desc& d = m->d;
  const LayerParams& p = m->lp[0];
  const LayerSaved& sv = m->ls[0];
  const int64_t T = m->T;
  MOSAIC_TRY(launch_linear_act_fwd(s, q, d.dtype, MOSAIC_GELU, T, d.in_dim, d.out_dim, x, P(m, p.w_1), P(m, p.b_1), W(m, sv.z), W(m, sv.a)));
  MOSAIC_TRY(launch_gemm(s, q, d.dtype, true, false, T, d.out_dim, d.out_dim, W(m, sv.a), d.out_dim, P(m, p.w_2), d.out_dim, y, d.out_dim, P(m, p.b_2), nullptr));
  return MOSAIC_OK;
}

mosaic_status projector_backward(mosaic_module* m, hipStream_t s, int q, const void* dy, void* dx) {
  const mosaic_module_desc& d = m->d;
  const LayerParams& p = m->lp[0];
  const LayerSaved& sv = m->ls[0];
  const int64_t T = m->T, no = d.out_dim, ni = d.in_dim;
  const int dt = d.dtype;
  void* dA = W(m, m->s_dA); void* dZ = W(m, m->s_dZ); void* csc = W(m, m->s_colsum);
  MOSAIC_TRY(launch_gemm(s, q, dt, true, true, T, no, no, dy, no, P(m, p.w_2), no, dA, no, nullptr, nullptr));
  MOSAIC_TRY(launch_gemm(s, q, dt, false, false, no, no, T, W(m, sv.a), no, dy, no, G(m, p.w_2), no, nullptr, nullptr, W(m, m->s_splitk)));
  MOSAIC_TRY(launch_colsum(s, q, dt, T, no, dy, G(m, p.b_2), csc));
  MOSAIC_TRY(launch_gelu_bwd_colsum(s, q, dt, T, no, W(m, sv.z), dA, dZ, G(m, p.b_1), csc));
  MOSAIC_TRY(launch_gemm(s, q, dt, false, false, ni, no, T, m->last_x, ni, dZ, no, G(m, p.w_1), no, nullptr, nullptr, W(m, m->s_splitk)));
  if (dx) MOSAIC_TRY(launch_gemm(s, q, dt, true, true, T, ni, no, dZ, no, P(m, p.w_1), no, dx, ni, nullptr, nullptr));
  return MOSAIC_OK;
}

// -------------------------------------------------------------------------- stems
mosaic_status patch_stem_forward(mosaic_module* m, hipStream_t s, int q, const void* x, void* y) {
  const mosaic_module_desc& d = m->d;
  const LayerParams& p = m->lp[0];
  const void* tokens = x;
  if (d.patch > 0) {
    const int side = (int)lround(sqrt((double)d.seq)) * d.patch;
    MOSAIC_TRY(launch_unfold(s, q, d.dtype, d.batch, side, d.patch, x, W(m, m->s_patches)));
    tokens = W(m, m->s_patches);
  }
  MOSAIC_TRY(launch_gemm(s, q, d.dtype, true, false, m->T, d.hidden, d.in_dim, tokens, d.in_dim, P(m, p.w_1), d.hidden, y, d.hidden, P(m, p.b_1), nullptr));
  MOSAIC_TRY(launch_add_pos(s, q, d.dtype, d.batch, d.seq, d.hidden, P(m, p.w_2), y));
  return MOSAIC_OK;
}

mosaic_status patch_stem_backward(mosaic_module* m, hipStream_t s, int q, const void* dy, void* dx) {
  const mosaic_module_desc& d = m->d;
  const LayerParams& p = m->lp[0];
  if (dx) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "the patch stem has no input gradient");
  const void* tokens = d.patch > 0 ? W(m, m->s_patches) : m->last_x;
  MOSAIC_TRY(launch_gemm(s, q, d.dtype, false, false, d.in_dim, d.hidden, m->T, tokens, d.in_dim, dy, d.hidden, G(m, p.w_1), d.hidden, nullptr, nullptr, W(m, m->s_splitk)));
  MOSAIC_TRY(launch_colsum(s, q, d.dtype, m->T, d.hidden, dy, G(m, p.b_1), W(m, m->s_colsum)));
  MOSAIC_TRY(launch_pos_grad(s, q, d.dtype, d.batch, d.seq, d.hidden, dy, G(m, p.w_2)));
  return MOSAIC_OK;
}

// conv stem: each convolution is a three-tap gather followed by a linear layer
mosaic_status conv_stem_forward(mosaic_module* m, hipStream_t s, int q, const void* x, void* y) {
  const mosaic_module_desc& d = m->d;
  const LayerParams& p = m->lp[0];
  const int dt = d.dtype, C = d.in_dim, h = d.hidden, Lo = d.seq, L = 2 * d.seq;
  const int64_t T = m->T, Tin = 2 * T;
  MOSAIC_TRY(launch_im2col1d(s, q, dt, d.batch, L, L, C, 1, x, W(m, m->c_p1)));
  MOSAIC_TRY(launch_linear_act_fwd(s, q, dt, MOSAIC_GELU, Tin, 3 * C, h, W(m, m->c_p1), P(m, p.w_1), P(m, p.b_1), W(m, m->c_z1), W(m, m->c_a1)));
  MOSAIC_TRY(launch_im2col1d(s, q, dt, d.batch, L, Lo, h, 2, W(m, m->c_a1), W(m, m->c_p2)));
  MOSAIC_TRY(launch_linear_act_fwd(s, q, dt, MOSAIC_GELU, T, 3 * h, h, W(m, m->c_p2), P(m, p.w_2), P(m, p.b_2), W(m, m->c_z2), y));
  MOSAIC_TRY(launch_add_pos(s, q, dt, d.batch, Lo, h, P(m, p.w_o), y));
  return MOSAIC_OK;
}

mosaic_status conv_stem_backward(mosaic_module* m, hipStream_t s, int q, const void* dy, void* dx) {
  const mosaic_module_desc& d = m->d;
  const LayerParams& p = m->lp[0];
  const int dt = d.dtype, C = d.in_dim, h = d.hidden, Lo = d.seq, L = 2 * d.seq;
  const int64_t T = m->T, Tin = 2 * T;
  void* csc = W(m, m->s_colsum); void* sk = W(m, m->s_splitk);
  MOSAIC_TRY(launch_pos_grad(s, q, dt, d.batch, Lo, h, dy, G(m, p.w_o)));
  MOSAIC_TRY(launch_gelu_bwd_colsum(s, q, dt, T, h, W(m, m->c_z2), dy, W(m, m->c_dz2), G(m, p.b_2), csc));
  MOSAIC_TRY(launch_gemm(s, q, dt, false, false, 3 * h, h, T, W(m, m->c_p2), 3 * h, W(m, m->c_dz2), h, G(m, p.w_2), h, nullptr, nullptr, sk));
  MOSAIC_TRY(launch_gemm(s, q, dt, true, true, T, 3 * h, h, W(m, m->c_dz2), h, P(m, p.w_2), h, W(m, m->c_dp2), 3 * h, nullptr, nullptr));
  MOSAIC_TRY(launch_col2im1d(s, q, dt, d.batch, L, Lo, h, 2, W(m, m->c_dp2), W(m, m->c_da1)));
  MOSAIC_TRY(launch_gelu_bwd_colsum(s, q, dt, Tin, h, W(m, m->c_z1), W(m, m->c_da1), W(m, m->c_dz1), G(m, p.b_1), csc));
  MOSAIC_TRY(launch_gemm(s, q, dt, false, false, 3 * C, h, Tin, W(m, m->c_p1), 3 * C, W(m, m->c_dz1), h, G(m, p.w_1), h, nullptr, nullptr, sk));
  if (dx) {
    MOSAIC_TRY(launch_gemm(s, q, dt, true, true, Tin, 3 * C, h, W(m, m->c_dz1), h, P(m, p.w_1), h, W(m, m->c_dp1), 3 * C, nullptr, nullptr));
    MOSAIC_TRY(launch_col2im1d(s, q, dt, d.batch, L, L, C, 1, W(m, m->c_dp1), dx));
  }
  return MOSAIC_OK;
}

}  // namespace

// ================================================================== C ABI: modules
extern "C" {

mosaic_status mosaic_module_create(const mosaic_module_desc* desc, mosaic_module** out) {
  if (!desc || !out) MOSAIC_FAIL(MOSAIC_EINVAL, "null argument");
  *out = nullptr;
  MOSAIC_TRY(validate(*desc));
  mosaic_module* m = new (std::nothrow) mosaic_module();
  if (!m) MOSAIC_FAIL(MOSAIC_ENOMEM, "host allocation failed");
  m->d = *desc;
  m->esize = dtype_size(desc->dtype);
  m->T = (int64_t)desc->batch * desc->seq;
  if (desc->kind == MOSAIC_PROJECTOR || desc->kind >= MOSAIC_PATCH_STEM) m->d.layers = 1;
  build_layout(m);
  *out = m;
  return MOSAIC_OK;
}

mosaic_status mosaic_module_destroy(mosaic_module* m) {
  delete m;
  return MOSAIC_OK;
}

size_t mosaic_module_param_bytes(const mosaic_module* m) { return m ? (size_t)m->param_elems * m->esize : 0; }
size_t mosaic_module_workspace_bytes(const mosaic_module* m) { return m ? m->ws_bytes : 0; }

size_t mosaic_module_input_elems(const mosaic_module* m) {
  if (!m) return 0;
  const mosaic_module_desc& d = m->d;
  switch (d.kind) {
    case MOSAIC_PROJECTOR: return (size_t)m->T * d.in_dim;
    case MOSAIC_PATCH_STEM: return (size_t)m->T * d.in_dim;   // unfolding permutes, never drops, pixels
    case MOSAIC_TEXT_STEM: return (size_t)d.batch * d.n_img * d.hidden;
    case MOSAIC_CONV_STEM: return (size_t)2 * m->T * d.in_dim;   // twice as many input frames as output tokens
    default: return (size_t)m->T * d.hidden;
  }
}

size_t mosaic_module_output_elems(const mosaic_module* m) {
  if (!m) return 0;
  return (size_t)m->T * (m->d.kind == MOSAIC_PROJECTOR ? m->d.out_dim : m->d.hidden);
}

int32_t mosaic_module_tensor_count(const mosaic_module* m) { return m ? (int32_t)m->tensors.size() : 0; }

mosaic_status mosaic_module_tensor_info(const mosaic_module* m, int32_t i, char* name32, int64_t* offset,
                                        int64_t* rows, int64_t* cols) {
  if (!m) MOSAIC_FAIL(MOSAIC_EINVAL, "null module");
  if (i < 0 || i >= (int32_t)m->tensors.size()) MOSAIC_FAIL(MOSAIC_EINVAL, "tensor index %d out of range", i);
  const TensorInfo& t = m->tensors[i];
  if (name32) { strncpy(name32, t.name.c_str(), 31); name32[31] = 0; }
  if (offset) *offset = t.offset;
  if (rows) *rows = t.rows;
  if (cols) *cols = t.cols;
  return MOSAIC_OK;
}

mosaic_status mosaic_module_bind(mosaic_module* m, void* params, void* grads, void* workspace, size_t workspace_bytes) {
  if (!m || !params || !grads || !workspace) MOSAIC_FAIL(MOSAIC_EINVAL, "null argument");
  if (workspace_bytes < m->ws_bytes)
    MOSAIC_FAIL(MOSAIC_ENOMEM, "workspace of %zu bytes is smaller than the %zu required", workspace_bytes, m->ws_bytes);
  if (((uintptr_t)workspace % 256) || ((uintptr_t)params % 16) || ((uintptr_t)grads % 16))
    MOSAIC_FAIL(MOSAIC_EINVAL, "workspace must be 256-byte aligned, params and grads 16-byte aligned");
  m->params = (char*)params; m->grads = (char*)grads; m->ws = (char*)workspace;
  m->forward_done = false;
  return MOSAIC_OK;
}

mosaic_status mosaic_module_bind_ids(mosaic_module* m, const int32_t* ids) {
  if (!m || !ids) MOSAIC_FAIL(MOSAIC_EINVAL, "null argument");
  if (m->d.kind != MOSAIC_TEXT_STEM) MOSAIC_FAIL(MOSAIC_EINVAL, "only a text stem takes token ids");
  m->ids = ids;
  return MOSAIC_OK;
}

mosaic_status mosaic_module_bind_image_counts(mosaic_module* m, const int32_t* counts) {
  if (!m) MOSAIC_FAIL(MOSAIC_EINVAL, "null argument");
  if (m->d.kind != MOSAIC_TEXT_STEM) MOSAIC_FAIL(MOSAIC_EINVAL, "only a text stem takes image-token counts");
  m->img_counts = counts;        // NULL: back to n_img image tokens for every sample
  return MOSAIC_OK;
}

static mosaic_status resolve_quota(int32_t quota, const mosaic_stream* stream, int* q) {
  DeviceInfo di;
  MOSAIC_TRY(mosaic_device_info(&di));
  if (quota <= 0 || quota > di.cu_count) MOSAIC_FAIL(MOSAIC_EQUOTA, "quota %d outside [1, %d]", quota, di.cu_count);
  if (stream && mosaic_stream_quota_or(stream, quota) != quota)
    MOSAIC_FAIL(MOSAIC_EQUOTA, "quota %d differs from the stream's quota %d", quota, mosaic_stream_quota_or(stream, quota));
  *q = quota;
  return MOSAIC_OK;
}

mosaic_status mosaic_module_forward(mosaic_module* m, int32_t quota, const mosaic_stream* stream, const void* x, void* y) {
  MOSAIC_TRY(check_bound(m));
  if (!x || !y) MOSAIC_FAIL(MOSAIC_EINVAL, "null activation pointer");
  int q;
  MOSAIC_TRY(resolve_quota(quota, stream, &q));
  hipStream_t s = mosaic_stream_hip(stream);
  m->last_x = x;
  mosaic_status st;
  switch (m->d.kind) {
    case MOSAIC_ENCODER:
    case MOSAIC_DECODER: st = layers_forward(m, s, q, x, y); break;
    case MOSAIC_PROJECTOR: st = projector_forward(m, s, q, x, y); break;
    case MOSAIC_PATCH_STEM: st = patch_stem_forward(m, s, q, x, y); break;
    case MOSAIC_CONV_STEM: st = conv_stem_forward(m, s, q, x, y); break;
    default:
      if (!m->ids) MOSAIC_FAIL(MOSAIC_EINVAL, "text stem has no token ids bound");
      st = launch_text_stem_fwd(s, q, m->d.dtype, m->d.batch, m->d.seq, m->d.n_img, m->d.hidden, m->d.vocab, x, m->ids, m->img_counts, P(m, m->lp[0].w_1), y);
  }
  m->forward_done = (st == MOSAIC_OK);
  return st;
}

mosaic_status mosaic_module_backward(mosaic_module* m, int32_t quota, const mosaic_stream* stream, const void* dy, void* dx) {
  MOSAIC_TRY(check_bound(m));
  if (!dy) MOSAIC_FAIL(MOSAIC_EINVAL, "null upstream gradient");
  if (!m->forward_done) MOSAIC_FAIL(MOSAIC_EINVAL, "backward called before forward");
  int q;
  MOSAIC_TRY(resolve_quota(quota, stream, &q));
  hipStream_t s = mosaic_stream_hip(stream);
  switch (m->d.kind) {
    case MOSAIC_ENCODER:
    case MOSAIC_DECODER: return layers_backward(m, s, q, dy, dx);
    case MOSAIC_PROJECTOR: return projector_backward(m, s, q, dy, dx);
    case MOSAIC_PATCH_STEM: return patch_stem_backward(m, s, q, dy, dx);
    case MOSAIC_CONV_STEM: return conv_stem_backward(m, s, q, dy, dx);
    default:
      return launch_text_stem_bwd(s, q, m->d.dtype, m->d.batch, m->d.seq, m->d.n_img, m->d.hidden, m->d.vocab, dy, m->ids, m->img_counts, dx, G(m, m->lp[0].w_1));
  }
}

mosaic_status mosaic_module_step(mosaic_module* m, int32_t quota, const mosaic_stream* stream, const void* x,
                                 const void* dy, const void* target, void* y, void* dx, float* loss) {
  MOSAIC_TRY(check_bound(m));
  if ((dy == nullptr) == (target == nullptr)) MOSAIC_FAIL(MOSAIC_EINVAL, "exactly one of dy and target must be given");
  if (target && !loss) MOSAIC_FAIL(MOSAIC_EINVAL, "a target needs a loss output");
  MOSAIC_TRY(mosaic_module_forward(m, quota, stream, x, y));
  const void* g = dy;
  if (target) {
    hipStream_t s = mosaic_stream_hip(stream);
    MOSAIC_TRY(launch_mse(s, quota, m->d.dtype, (int64_t)mosaic_module_output_elems(m), y, target, W(m, m->s_dyloss), loss, W(m, m->s_mse)));
    g = W(m, m->s_dyloss);
  }
  return mosaic_module_backward(m, quota, stream, g, dx);
}

size_t mosaic_module_optimizer_state_bytes(const mosaic_module* m, int32_t use_master) {
  return m ? (size_t)m->param_elems * sizeof(float) * (use_master ? 3 : 2) : 0;
}

mosaic_status mosaic_module_adamw_step(mosaic_module* m, int32_t quota, const mosaic_stream* stream, void* state,
                                       size_t state_bytes, int32_t use_master, float lr, float beta1, float beta2,
                                       float eps, float weight_decay, int64_t step) {
  MOSAIC_TRY(check_bound(m));
  if (!state) MOSAIC_FAIL(MOSAIC_EINVAL, "null optimizer state");
  if (state_bytes < mosaic_module_optimizer_state_bytes(m, use_master)) MOSAIC_FAIL(MOSAIC_ENOMEM, "optimizer state too small");
  if ((uintptr_t)state % 16) MOSAIC_FAIL(MOSAIC_EINVAL, "optimizer state must be 16-byte aligned");
  int q;
  MOSAIC_TRY(resolve_quota(quota, stream, &q));
  float* mom = (float*)state;
  float* var = mom + m->param_elems;
  float* master = use_master ? var + m->param_elems : nullptr;
  // one launch over the flat buffer: every tensor starts on a 16-byte boundary and the padding
  // between tensors holds zeros with zero gradients, which the update leaves at zero
  return launch_adamw(mosaic_stream_hip(stream), q, m->d.dtype, m->param_elems, m->params, m->grads, mom, var, master,
                      lr, beta1, beta2, eps, weight_decay, step);
}

}  // extern "C"
