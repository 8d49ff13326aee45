// Layer and epoch orchestration: the order rule (section "Order of Computation"), the
// activation buffer plan (section "Memory Optimizations") and the forward / backward chains
// of Eq. 5-11, all enqueued on one stream.
//
// Buffer plan on one GPU: one result buffer per layer (holds the layer output H', later the
// gradient with respect to it, in place) plus one temporary shared by all layers (HW in the
// forward pass, the SpMM result HW_G in the backward pass).  The two broadcast buffers of the
// paper's multi-GPU scheme have no counterpart here.  A layer that runs SpMM first keeps its
// A^ H product for the weight gradient instead of recomputing it: with 288 GB of HBM that one
// extra buffer is cheaper than one more SpMM per epoch.
#include "common.h"
#include "graph.h"

#include <algorithm>
#include <new>
#include <vector>

struct mggcn_model {
  const mggcn_graph* g = nullptr;
  int32_t n = 0, L = 0;
  std::vector<int32_t> dims, orders;
  std::vector<int64_t> ld_act;       // leading dimension of layer l's result buffer
  std::vector<size_t> off_act;       // arena offsets
  std::vector<size_t> off_p;         // A^ H buffer of SpMM-first layers ((size_t)-1 otherwise)
  std::vector<int64_t> ld_p;
  size_t off_tmp = 0, off_gemm_ws = 0, off_loss_ws = 0;
  size_t gemm_ws_bytes = 0, loss_ws_bytes = 0, arena_bytes = 0;
  char* arena = nullptr;
  bool cache_input = false;  // layer 0 works from a stored A^ X
  bool cache_valid = false;
  bool gather_bf16 = false;  // every SpMM gathers a bfloat16 copy of its operand
  size_t off_bf16 = 0;       // that copy: n x padded_ld_bf16(widest SpMM) 2-byte elements
  int32_t bf16_width = 0;    // the widest SpMM operand it was sized for
  bool gemm_pieces = false;  // MGGCN_MODEL_GEMM_BF16X3
};

namespace mggcn {
namespace {

// Rows of the model's own buffers start at multiples of 64 bytes (32 for rows that short): a row
// then never touches more 128-byte lines than its length requires -- a gather costs time per line,
// and bfloat16 rows of 41 or 47 elements at multiples of 32 bytes measured 25-30 % slower -- and
// every row is aligned for the widest loads.
int64_t padded_ld(int32_t width) { return (int64_t)align_up((size_t)std::max(width, 1), 16); }
int64_t padded_ld_bf16(int32_t width) { return width <= 16 ? 16 : (int64_t)align_up((size_t)width, 32); }

int resolve_order(int32_t d_in, int32_t d_out, int32_t requested) {
  if (requested == MGGCN_ORDER_GEMM_FIRST || requested == MGGCN_ORDER_SPMM_FIRST) return requested;
  return d_in < d_out ? MGGCN_ORDER_SPMM_FIRST : MGGCN_ORDER_GEMM_FIRST;
}

// The SpMM of a layer: straight from the fp32 operand, or (model flag) from a bfloat16 copy of it
// made just before, which halves the bytes the product gathers.
int gathered_spmm(const mggcn_model* m, int op, const float* X, int64_t ldx, int32_t F, int epi, float* Y,
                  int64_t ldy, void* stream) {
  if (!m->gather_bf16) return mggcn_spmm(m->g, op, X, ldx, F, 0.f, epi, Y, ldy, stream);
  uint16_t* Xb = reinterpret_cast<uint16_t*>(m->arena + m->off_bf16);
  const int64_t ldb = padded_ld_bf16(F);
  const int rc = mggcn_f32_to_bf16(m->n, F, X, ldx, Xb, ldb, stream);
  if (rc) return rc;
  return mggcn_spmm_bf16(m->g, op, Xb, ldb, F, 0.f, epi, Y, ldy, stream);
}

int check_layer(const mggcn_model* m, int32_t l) {
  MGGCN_REQUIRE(m != nullptr, MGGCN_E_INVALID_ARG, "model is NULL");
  MGGCN_REQUIRE(l >= 0 && l < m->L, MGGCN_E_INVALID_ARG, "layer %d outside [0, %d)", l, m->L);
  MGGCN_REQUIRE(m->arena != nullptr, MGGCN_E_WORKSPACE, "model is not bound to an arena");
  return MGGCN_OK;
}

}  // namespace
}  // namespace mggcn

using namespace mggcn;

extern "C" {

int32_t mggcn_model_spmm_width_max(const int32_t* dims, const int32_t* orders, int32_t L, int32_t flags) {
  if (!dims || L < 1) return 0;
  int32_t w = 0;
  for (int32_t l = 0; l < L; ++l) {
    int o = resolve_order(dims[l], dims[l + 1], orders ? orders[l] : MGGCN_ORDER_AUTO);
    if (l == 0 && (flags & MGGCN_MODEL_CACHE_INPUT)) o = MGGCN_ORDER_SPMM_FIRST;
    w = std::max(w, o == MGGCN_ORDER_SPMM_FIRST ? dims[l] : dims[l + 1]);
  }
  return w;
}

int mggcn_model_create(const mggcn_graph* g, int32_t L, const int32_t* dims, const int32_t* orders,
                       int32_t flags, mggcn_model** out) {
  MGGCN_REQUIRE(out != nullptr, MGGCN_E_INVALID_ARG, "out is NULL");
  *out = nullptr;
  MGGCN_REQUIRE(g != nullptr && dims != nullptr, MGGCN_E_INVALID_ARG, "graph / dims is NULL");
  MGGCN_REQUIRE(L >= 1 && L <= 64, MGGCN_E_INVALID_ARG, "layer count %d outside [1, 64]", L);
  MGGCN_REQUIRE((flags & ~(MGGCN_MODEL_CACHE_INPUT | MGGCN_MODEL_GATHER_BF16 | MGGCN_MODEL_GEMM_BF16X3)) == 0, MGGCN_E_INVALID_ARG,
                "unknown model flags 0x%x", flags);
  MGGCN_REQUIRE(g->fwd.n_rows == g->fwd.n_cols, MGGCN_E_INVALID_ARG,
                "a model needs a square graph, got %d x %d", g->fwd.n_rows, g->fwd.n_cols);
  for (int32_t l = 0; l <= L; ++l)
    MGGCN_REQUIRE(dims[l] >= 1, MGGCN_E_INVALID_ARG, "dims[%d] = %d must be positive", l, dims[l]);
  if (orders)
    for (int32_t l = 0; l < L; ++l)
      MGGCN_REQUIRE(orders[l] >= MGGCN_ORDER_AUTO && orders[l] <= MGGCN_ORDER_SPMM_FIRST,
                    MGGCN_E_INVALID_ARG, "orders[%d] = %d is not an mggcn_order", l, orders[l]);
  mggcn_model* m = new (std::nothrow) mggcn_model;
  MGGCN_REQUIRE(m != nullptr, MGGCN_E_NO_MEMORY, "out of host memory");
  const int rc = guarded([&]() -> int {
    m->g = g;
    m->n = g->fwd.n_rows;
    m->L = L;
    m->cache_input = (flags & MGGCN_MODEL_CACHE_INPUT) != 0;
    m->gather_bf16 = (flags & MGGCN_MODEL_GATHER_BF16) != 0;
    m->gemm_pieces = (flags & MGGCN_MODEL_GEMM_BF16X3) != 0;
    m->dims.assign(dims, dims + L + 1);
    m->orders.resize(L);
    m->ld_act.resize(L);
    m->off_act.resize(L);
    m->off_p.assign(L, (size_t)-1);
    m->ld_p.assign(L, 0);
    const size_t n = (size_t)std::max(m->n, 1);
    size_t off = 0;
    int32_t tmp_width = 1;
    for (int32_t l = 0; l < L; ++l) {
      m->orders[l] = resolve_order(dims[l], dims[l + 1], orders ? orders[l] : MGGCN_ORDER_AUTO);
      if (l == 0 && m->cache_input) m->orders[l] = MGGCN_ORDER_SPMM_FIRST;  // its A^ H buffer is the cache
      m->ld_act[l] = padded_ld(dims[l + 1]);
      m->off_act[l] = off;
      off += align_up(n * (size_t)m->ld_act[l] * sizeof(float), kWsAlign);
      if (m->orders[l] == MGGCN_ORDER_SPMM_FIRST) {
        m->ld_p[l] = padded_ld(dims[l]);
        m->off_p[l] = off;
        off += align_up(n * (size_t)m->ld_p[l] * sizeof(float), kWsAlign);
        if (!(l == 0 && m->cache_input)) tmp_width = std::max(tmp_width, dims[l]);
      } else {
        tmp_width = std::max(tmp_width, dims[l + 1]);
      }
      m->gemm_ws_bytes = std::max(
          m->gemm_ws_bytes, mggcn_gemm_workspace_bytes(MGGCN_OP_T, MGGCN_OP_N, dims[l], dims[l + 1], m->n));
    }
    m->off_tmp = off;
    off += align_up(n * (size_t)padded_ld(tmp_width) * sizeof(float), kWsAlign);
    if (m->gather_bf16) {
      const int32_t w = mggcn_model_spmm_width_max(dims, m->orders.data(), L, flags);
      m->off_bf16 = off;
      m->bf16_width = w;
      off += align_up(n * (size_t)padded_ld_bf16(w) * sizeof(uint16_t), kWsAlign);
    }
    m->off_gemm_ws = off;
    off += align_up(m->gemm_ws_bytes, kWsAlign);
    m->loss_ws_bytes = mggcn_softmax_ce_workspace_bytes(m->n);
    m->off_loss_ws = off;
    off += align_up(m->loss_ws_bytes, kWsAlign);
    m->arena_bytes = off + kWsAlign;
    return MGGCN_OK;
  });
  if (rc) { delete m; return rc; }
  *out = m;
  return MGGCN_OK;
}

int mggcn_model_destroy(mggcn_model* m) {
  delete m;
  return MGGCN_OK;
}

size_t mggcn_model_arena_bytes(const mggcn_model* m) { return m ? m->arena_bytes : 0; }

int mggcn_model_bind(mggcn_model* m, void* arena, size_t arena_bytes) {
  MGGCN_REQUIRE(m != nullptr, MGGCN_E_INVALID_ARG, "model is NULL");
  MGGCN_REQUIRE(arena && aligned(arena, kWsAlign), MGGCN_E_WORKSPACE, "arena is NULL or not 256-byte aligned");
  MGGCN_REQUIRE(arena_bytes >= m->arena_bytes, MGGCN_E_WORKSPACE, "arena too small: %zu bytes given, %zu needed",
                arena_bytes, m->arena_bytes);
  m->arena = static_cast<char*>(arena);
  m->cache_valid = false;
  return MGGCN_OK;
}

int mggcn_model_cache_input(mggcn_model* m, const float* X, int64_t ldx, void* stream) {
  MGGCN_REQUIRE(m != nullptr, MGGCN_E_INVALID_ARG, "model is NULL");
  MGGCN_REQUIRE(m->cache_input, MGGCN_E_INVALID_ARG, "model was created without MGGCN_MODEL_CACHE_INPUT");
  MGGCN_REQUIRE(m->arena != nullptr, MGGCN_E_WORKSPACE, "model is not bound to an arena");
  MGGCN_REQUIRE(X != nullptr && ldx >= m->dims[0], MGGCN_E_INVALID_ARG, "X is NULL or ldx < d_0");
  float* P = reinterpret_cast<float*>(m->arena + m->off_p[0]);
  const int rc = gathered_spmm(m, MGGCN_OP_N, X, ldx, m->dims[0], MGGCN_EPI_NONE, P, m->ld_p[0], stream);
  if (rc) return rc;
  m->cache_valid = true;
  return MGGCN_OK;
}

int mggcn_model_order(const mggcn_model* m, int32_t l) {
  MGGCN_REQUIRE(m != nullptr, MGGCN_E_INVALID_ARG, "model is NULL");
  MGGCN_REQUIRE(l >= 0 && l < m->L, MGGCN_E_INVALID_ARG, "layer %d outside [0, %d)", l, m->L);
  return m->orders[l];
}

int mggcn_model_activation(const mggcn_model* m, int32_t l, float** ptr_out, int64_t* ld_out) {
  int rc = check_layer(m, l);
  if (rc) return rc;
  MGGCN_REQUIRE(ptr_out && ld_out, MGGCN_E_INVALID_ARG, "ptr_out / ld_out is NULL");
  *ptr_out = reinterpret_cast<float*>(m->arena + m->off_act[l]);
  *ld_out = m->ld_act[l];
  return MGGCN_OK;
}

int mggcn_model_gather_operand(const mggcn_model* m, int32_t width, uint16_t** ptr_out, int64_t* ld_out) {
  MGGCN_REQUIRE(m != nullptr && ptr_out && ld_out, MGGCN_E_INVALID_ARG, "model / ptr_out / ld_out is NULL");
  MGGCN_REQUIRE(m->gather_bf16, MGGCN_E_INVALID_ARG, "model was created without MGGCN_MODEL_GATHER_BF16");
  MGGCN_REQUIRE(m->arena != nullptr, MGGCN_E_WORKSPACE, "model is not bound to an arena");
  MGGCN_REQUIRE(width >= 1 && width <= m->bf16_width, MGGCN_E_INVALID_ARG,
                "width %d outside [1, %d], the widths of this model's SpMM operands", width, m->bf16_width);
  *ptr_out = reinterpret_cast<uint16_t*>(m->arena + m->off_bf16);
  *ld_out = padded_ld_bf16(width);
  return MGGCN_OK;
}

int mggcn_layer_fwd(mggcn_model* m, int32_t l, const float* H_in, int64_t ld_in, const float* W,
                    int64_t ldw, int relu, float* H_out, int64_t ld_out, void* stream) {
  int rc = check_layer(m, l);
  if (rc) return rc;
  const int32_t d_in = m->dims[l], d_out = m->dims[l + 1];
  const bool cached = l == 0 && m->cache_input;
  MGGCN_REQUIRE(!cached || m->cache_valid, MGGCN_E_INVALID_ARG,
                "mggcn_model_cache_input has not been called since the model was bound");
  MGGCN_REQUIRE((cached || H_in) && W && H_out, MGGCN_E_INVALID_ARG, "H_in / W / H_out is NULL");
  MGGCN_REQUIRE((cached || ld_in >= d_in) && ldw >= d_out && ld_out >= d_out, MGGCN_E_INVALID_ARG,
                "leading dimension too small for layer %d (%d -> %d)", l, d_in, d_out);
  const int epi = relu ? MGGCN_EPI_RELU : MGGCN_EPI_NONE;
  float* tmp = reinterpret_cast<float*>(m->arena + m->off_tmp);
  if (m->orders[l] == MGGCN_ORDER_GEMM_FIRST) {
    // Eq. 5 then Eq. 6-7:  HW = H W ;  H' = relu(A^ HW)
    const int64_t ldt = padded_ld(d_out);
    rc = gemm_run(m->gemm_pieces, MGGCN_OP_N, MGGCN_OP_N, m->n, d_out, d_in, H_in, ld_in, W, ldw, 0.f, MGGCN_EPI_NONE, tmp,
                    ldt, nullptr, 0, stream);
    if (rc) return rc;
    return gathered_spmm(m, MGGCN_OP_N, tmp, ldt, d_out, epi, H_out, ld_out, stream);
  }
  // associativity:  P = A^ H ;  H' = relu(P W)
  float* P = reinterpret_cast<float*>(m->arena + m->off_p[l]);
  if (!cached) {
    rc = gathered_spmm(m, MGGCN_OP_N, H_in, ld_in, d_in, MGGCN_EPI_NONE, P, m->ld_p[l], stream);
    if (rc) return rc;
  }
  return gemm_run(m->gemm_pieces, MGGCN_OP_N, MGGCN_OP_N, m->n, d_out, d_in, P, m->ld_p[l], W, ldw, 0.f, epi, H_out, ld_out,
                    nullptr, 0, stream);
}

int mggcn_layer_bwd(mggcn_model* m, int32_t l, const float* H_in, int64_t ld_in, const float* act,
                    int64_t ld_act, float* G, int64_t ldg, const float* W, int64_t ldw, float* W_G,
                    int64_t ldwg, float* H_G, int64_t ldhg, int hg_relu_mask, void* stream) {
  int rc = check_layer(m, l);
  if (rc) return rc;
  const int32_t d_in = m->dims[l], d_out = m->dims[l + 1];
  const bool cached = l == 0 && m->cache_input;
  MGGCN_REQUIRE(!cached || m->cache_valid, MGGCN_E_INVALID_ARG,
                "mggcn_model_cache_input has not been called since the model was bound");
  MGGCN_REQUIRE((cached || H_in) && G && W && W_G, MGGCN_E_INVALID_ARG, "H_in / G / W / W_G is NULL");
  MGGCN_REQUIRE((cached || ld_in >= d_in) && ldg >= d_out && ldw >= d_out && ldwg >= d_out, MGGCN_E_INVALID_ARG,
                "leading dimension too small for layer %d (%d -> %d)", l, d_in, d_out);
  MGGCN_REQUIRE(!act || ld_act >= d_out, MGGCN_E_INVALID_ARG, "ld_act < %d", d_out);
  MGGCN_REQUIRE(!H_G || ldhg >= d_in, MGGCN_E_INVALID_ARG, "ldhg < %d", d_in);
  MGGCN_REQUIRE(hg_relu_mask || H_G == nullptr || H_in == nullptr || H_G != H_in, MGGCN_E_INVALID_ARG,
                "H_G may alias H_in only with hg_relu_mask set");
  // The shared temporary is sized without d_0 for a cached first layer (U = Z_G W^T would need
  // n x d_0 of it): the input features take no gradient there.
  MGGCN_REQUIRE(!(cached && H_G), MGGCN_E_INVALID_ARG,
                "layer 0 of a MGGCN_MODEL_CACHE_INPUT model forms no gradient with respect to X: pass H_G = NULL");
  if (act) {  // Eq. 8, unfused
    rc = mggcn_relu_bwd(m->n, d_out, act, ld_act, G, ldg, stream);
    if (rc) return rc;
  }
  const int hg_epi = hg_relu_mask ? MGGCN_EPI_RELU_MASK : MGGCN_EPI_NONE;
  float* tmp = reinterpret_cast<float*>(m->arena + m->off_tmp);
  void* gws = m->arena + m->off_gemm_ws;
  if (m->orders[l] == MGGCN_ORDER_GEMM_FIRST) {
    // Eq. 9: T = A^^T Z_G ;  Eq. 10: W_G = H^T T ;  Eq. 11: H_G = T W^T
    const int64_t ldt = padded_ld(d_out);
    rc = gathered_spmm(m, MGGCN_OP_T, G, ldg, d_out, MGGCN_EPI_NONE, tmp, ldt, stream);
    if (rc) return rc;
    rc = gemm_run(m->gemm_pieces, MGGCN_OP_T, MGGCN_OP_N, d_in, d_out, m->n, H_in, ld_in, tmp, ldt, 0.f, MGGCN_EPI_NONE, W_G,
                    ldwg, gws, m->gemm_ws_bytes, stream);
    if (rc || !H_G) return rc;
    return gemm_run(m->gemm_pieces, MGGCN_OP_N, MGGCN_OP_T, m->n, d_in, d_out, tmp, ldt, W, ldw, 0.f, hg_epi, H_G, ldhg,
                      nullptr, 0, stream);
  }
  // SpMM-first association:  W_G = (A^ H)^T Z_G ;  U = Z_G W^T ;  H_G = A^^T U
  const float* P = reinterpret_cast<const float*>(m->arena + m->off_p[l]);
  rc = gemm_run(m->gemm_pieces, MGGCN_OP_T, MGGCN_OP_N, d_in, d_out, m->n, P, m->ld_p[l], G, ldg, 0.f, MGGCN_EPI_NONE, W_G,
                  ldwg, gws, m->gemm_ws_bytes, stream);
  if (rc || !H_G) return rc;
  const int64_t ldu = padded_ld(d_in);
  rc = gemm_run(m->gemm_pieces, MGGCN_OP_N, MGGCN_OP_T, m->n, d_in, d_out, G, ldg, W, ldw, 0.f, MGGCN_EPI_NONE, tmp, ldu,
                  nullptr, 0, stream);
  if (rc) return rc;
  return gathered_spmm(m, MGGCN_OP_T, tmp, ldu, d_in, hg_epi, H_G, ldhg, stream);
}

int mggcn_epoch(mggcn_model* m, const float* X, int64_t ldx, const int32_t* labels, const float* const* W,
                float* loss_dev, float* const* W_G, void* stream) {
  MGGCN_REQUIRE(m != nullptr, MGGCN_E_INVALID_ARG, "model is NULL");
  MGGCN_REQUIRE(m->arena != nullptr, MGGCN_E_WORKSPACE, "model is not bound to an arena");
  MGGCN_REQUIRE((X || m->cache_input) && labels && W && loss_dev && W_G, MGGCN_E_INVALID_ARG, "NULL argument");
  MGGCN_REQUIRE(m->cache_input || ldx >= m->dims[0], MGGCN_E_INVALID_ARG, "ldx %lld < d_0 %d", (long long)ldx,
                m->dims[0]);
  for (int32_t l = 0; l < m->L; ++l)
    MGGCN_REQUIRE(W[l] && W_G[l], MGGCN_E_INVALID_ARG, "W[%d] / W_G[%d] is NULL", l, l);
  const int32_t L = m->L;
  auto act = [&](int32_t l) { return reinterpret_cast<float*>(m->arena + m->off_act[l]); };

  const float* H = X;
  int64_t ldh = ldx;
  for (int32_t l = 0; l < L; ++l) {
    const int rc = mggcn_layer_fwd(m, l, H, ldh, W[l], m->dims[l + 1], l + 1 < L, act(l), m->ld_act[l], stream);
    if (rc) return rc;
    H = act(l);
    ldh = m->ld_act[l];
  }
  // the logits' buffer receives their gradient in place
  int rc = mggcn_softmax_ce(m->n, m->dims[L], act(L - 1), m->ld_act[L - 1], labels, loss_dev, act(L - 1),
                            m->ld_act[L - 1], m->arena + m->off_loss_ws, m->loss_ws_bytes, stream);
  if (rc) return rc;
  for (int32_t l = L - 1; l >= 0; --l) {
    // act(l) now holds the gradient of layer l's pre-activation (the ReLU' of Eq. 8 was fused
    // into whatever produced it); act(l-1) still holds H^(l) and is overwritten by its gradient.
    const float* H_in = l > 0 ? act(l - 1) : X;
    const int64_t ld_in = l > 0 ? m->ld_act[l - 1] : ldx;
    rc = mggcn_layer_bwd(m, l, H_in, ld_in, nullptr, 0, act(l), m->ld_act[l], W[l], m->dims[l + 1], W_G[l],
                         m->dims[l + 1], l > 0 ? act(l - 1) : nullptr, l > 0 ? m->ld_act[l - 1] : 0, 1, stream);
    if (rc) return rc;
  }
  return MGGCN_OK;
}

}  // extern "C"
