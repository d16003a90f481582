// C ABI of the library: argument checks, workspace carving, kernel sequencing.
// Every step of the layer runs in the kernels of gate.hip, dispatch_combine.hip
// and expert_gemm.hip; nothing here computes.
#include <mutex>
#include "common.h"

namespace {

using moe::align_up;

// Scratch memory of moe_gate_noalloc: one array per GPU, owned by the library's code object
// (it exists from the moment the library is loaded on a device until the process ends).
constexpr size_t kGateScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kGateScratchBytes];

// Device address of `scratch` on the current device.  In host code the array's name is only a
// stand-in for the symbol; its address on a device comes from hipGetSymbolAddress, once per
// device with that device current, and is kept.
constexpr int kScratchDevices = 64;
int gate_scratch_ptr(void** out) {
  static std::mutex lock;
  static void* ptr_of[kScratchDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kScratchDevices) return MOE_EHIP;
  std::lock_guard<std::mutex> guard(lock);
  if (ptr_of[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return MOE_EHIP;
    ptr_of[dev] = p;
  }
  *out = ptr_of[dev];
  return MOE_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_config(const moe_config* c) {
  if (c == nullptr) return MOE_EINVAL;
  if (c->G < 1 || c->S < 1 || c->M < 1 || c->H < 1 || c->E < 2 || c->C < 1) return MOE_EINVAL;
  if (c->act_dtype != MOE_F32 && c->act_dtype != MOE_BF16) return MOE_EINVAL;
  // rows are moved and multiplied in 16-byte pieces: 8 bf16 or 4 fp32 elements
  const int piece = c->act_dtype == MOE_F32 ? 4 : 8;
  if (c->M % piece != 0 || c->H % piece != 0) return MOE_EUNSUPPORTED;
  if ((long long)c->G * c->S > 0x3fffffffLL) return MOE_EUNSUPPORTED;
  if ((long long)c->E * c->G * c->C > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  return MOE_OK;
}

// Layout of the moe_forward workspace.
struct ForwardWs {
  size_t expert_idx, slot, weight, fill, src_token, c1, mean_gate, zero_row, packing, gates,
      signbits, buf, h, out, gate_ws, total;
};

// train: also the regions only the backward pass reads (softmax gates, relu sign bits)
ForwardWs carve(const moe_config& c, bool train) {
  const size_t N = (size_t)c.G * c.S, GE = (size_t)c.G * c.E, rows = (size_t)c.E * c.G * c.C;
  const size_t elt = c.act_dtype == MOE_F32 ? 4 : 2;
  ForwardWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  w.expert_idx = take(N * 2 * 4);
  w.slot = take(N * 2 * 4);
  w.weight = take(N * 2 * 4);
  w.fill = take(GE * 4);
  w.src_token = take(rows * 4);
  w.c1 = take(GE * 4);
  w.mean_gate = take(GE * 4);
  w.zero_row = take((size_t)c.M * elt);
  w.packing = take(moe::expert_ffn_can_pack(c) ? moe::row_packing_bytes(c) : 0);
  w.gates = take(train ? N * c.E * 4 : 0);
  w.signbits = take(train && moe::expert_gemm1_can_gather(c) ? moe::expert_signbits_bytes(c) : 0);
  w.buf = take(moe::expert_gemm1_can_gather(c) ? 0 : rows * c.M * elt);   // gathered from x instead
  w.h = take(rows * c.H * elt);
  w.out = take(rows * c.M * elt);
  w.gate_ws = take(moe::gate_workspace_bytes(c));
  w.total = off;
  return w;
}

// Layout of the moe_backward workspace.
struct BackwardWs {
  size_t dout, dh, dbuf, buf, dweight, dz, dzp, wgp, dxg, dwg_partial, total;
};

BackwardWs carve_bwd(const moe_config& c) {
  const size_t N = (size_t)c.G * c.S, rows = (size_t)c.E * c.G * c.C;
  const size_t elt = c.act_dtype == MOE_F32 ? 4 : 2;
  BackwardWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  w.dout = take(rows * c.M * elt);
  w.dh = take(rows * c.H * elt);
  w.dbuf = take(rows * c.M * elt);
  w.buf = take(rows * c.M * elt);
  w.dweight = take(N * 2 * 4);
  const moe::GateBwdPlan p = moe::gate_bwd_plan(c);
  w.dz = take(p.dz_bytes);
  w.dzp = take(p.dzp_bytes);
  w.wgp = take(p.wgp_bytes);
  w.dxg = take(p.dxg_bytes);
  w.dwg_partial = take(p.partial_bytes);
  w.total = off;
  return w;
}

int forward_impl(const moe_config* cfg, const void* x, const float* wg, const float* u,
                 const void* wi, const void* wo, void* y, float* aux, void* ws, size_t ws_bytes,
                 void* stream, void* const* events, bool keep_gates,
                 const void* wg_packed = nullptr) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {x, wg, u, wi, wo, y, aux, ws};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MOE_EINVAL;
  if (events != nullptr)
    for (int i = 0; i < MOE_FORWARD_EVENTS; ++i)
      if (events[i] == nullptr) return MOE_EINVAL;
  const ForwardWs w = carve(*cfg, keep_gates);
  if (ws_bytes < w.total) return MOE_EWORKSPACE;
  char* base = static_cast<char*>(ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  auto mark = [&](int i) {
    return events == nullptr ||
           hipEventRecord(static_cast<hipEvent_t>(events[i]), st) == hipSuccess;
  };
  int32_t* expert_idx = reinterpret_cast<int32_t*>(base + w.expert_idx);
  int32_t* slot = reinterpret_cast<int32_t*>(base + w.slot);
  float* weight = reinterpret_cast<float*>(base + w.weight);
  int32_t* src_token = reinterpret_cast<int32_t*>(base + w.src_token);
  // bf16 layers whose shape the persistent GEMM takes skip the dispatched buffer: the first
  // GEMM gathers its rows from x (then the dispatch mark coincides with the gate mark)
  const bool gather = moe::expert_gemm1_can_gather(*cfg);
  // ... and multiply only the occupied rows of each expert, packed to the front of its block
  const bool packed = moe::expert_ffn_can_pack(*cfg);
  const moe::RowPacking pk = moe::carve_row_packing(*cfg, base + w.packing);
  if (!mark(0)) return MOE_EHIP;
  rc = moe::launch_gate(*cfg, x, wg, u, expert_idx, slot, weight,
                        reinterpret_cast<int32_t*>(base + w.fill), src_token,
                        reinterpret_cast<int32_t*>(base + w.c1),
                        reinterpret_cast<float*>(base + w.mean_gate), aux,
                        keep_gates ? reinterpret_cast<float*>(base + w.gates) : nullptr,
                        base + w.gate_ws, gather ? base + w.zero_row : nullptr,
                        packed ? &pk : nullptr, wg_packed, st);
  if (rc != MOE_OK) return rc;
  if (!mark(1)) return MOE_EHIP;
  if (!gather) rc = moe::launch_dispatch(*cfg, x, src_token, base + w.buf, nullptr, st);
  if (rc != MOE_OK) return rc;
  if (!mark(2)) return MOE_EHIP;
  if (packed) {
    rc = moe::launch_expert_ffn_packed(*cfg, x, pk, base + w.zero_row, wi, wo, base + w.h,
                                       base + w.out, false, keep_gates ? base + w.signbits : nullptr,
                                       st, events != nullptr ? events[3] : nullptr);
    if (rc != MOE_OK) return rc;
  } else {
    rc = gather ? moe::launch_expert_gemm1_gather(*cfg, x, src_token, base + w.zero_row, wi,
                                                  base + w.h, keep_gates ? base + w.signbits : nullptr,
                                                  st)
                : moe::launch_expert_gemm1(*cfg, base + w.buf, wi, base + w.h, st);
    if (rc != MOE_OK) return rc;
    if (!mark(3)) return MOE_EHIP;
    rc = moe::launch_expert_gemm2(*cfg, base + w.h, wo, base + w.out, st);
    if (rc != MOE_OK) return rc;
  }
  if (!mark(4)) return MOE_EHIP;
  rc = moe::launch_combine(*cfg, base + w.out, expert_idx, slot, weight,
                           packed ? pk.row_base : nullptr, y, st);
  if (rc != MOE_OK) return rc;
  return mark(5) ? MOE_OK : MOE_EHIP;
}

// ---- encoder layers: C[rows,N] = A[rows,K] . B[K,N] (optionally relu) through the expert GEMM
// launchers with a one-expert configuration
int dense_gemm(const moe_config& c, long long rows, int K, int N, bool relu, const void* A,
               const void* B, void* Cout, hipStream_t st) {
  if (rows > 0x7fffffffLL) return MOE_EUNSUPPORTED;
  moe_config g = c;
  g.E = 1;
  g.G = 1;
  g.C = (int)rows;
  if (relu) {                       // h = relu(buf . wi): buf [rows, M:=K], wi [K, H:=N]
    g.M = K;
    g.H = N;
    return moe::launch_expert_gemm1(g, A, B, Cout, st);
  }
  g.M = N;                          // out = h . wo: h [rows, H:=K], wo [K, M:=N]
  g.H = K;
  return moe::launch_expert_gemm2(g, A, B, Cout, st);
}

int check_dims(const moe_config* cfg, const moe_encoder_dims* d) {
  if (d == nullptr) return MOE_EINVAL;
  if (d->B < 1 || d->L < 1 || d->heads < 1 || d->d < 1) return MOE_EINVAL;
  if ((long long)d->B * d->L != (long long)cfg->G * cfg->S) return MOE_EINVAL;
  if (d->d % 8 != 0 || (long long)d->heads * d->d > 0x7fffffLL) return MOE_EUNSUPPORTED;
  return MOE_OK;
}

struct AttentionWs { size_t qkv, ctx, total; };
AttentionWs carve_att(const moe_config& c, const moe_encoder_dims& d) {
  const size_t N = (size_t)c.G * c.S, A = (size_t)d.heads * d.d;
  const size_t elt = c.act_dtype == MOE_F32 ? 4 : 2;
  AttentionWs w{};
  w.qkv = 0;
  w.ctx = align_up(N * 3 * A * elt, 256);
  w.total = w.ctx + align_up(N * A * elt, 256);
  return w;
}

struct EncoderWs { size_t norm, sub, a, b, c, hden, att, moe, total; };
EncoderWs carve_enc(const moe_config& c, const moe_encoder_dims& d) {
  const size_t N = (size_t)c.G * c.S;
  const size_t elt = c.act_dtype == MOE_F32 ? 4 : 2;
  EncoderWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  w.norm = take(N * c.M * elt);
  w.sub = take(N * c.M * elt);
  w.a = take(N * c.M * elt);
  w.b = take(N * c.M * elt);
  w.c = take(N * c.M * elt);
  w.hden = take(N * c.H * elt);
  w.att = take(carve_att(c, d).total);
  w.moe = take(carve(c, false).total);
  w.total = off;
  return w;
}

int attention_impl(const moe_config& c, const moe_encoder_dims& d, const void* u, const void* wqkv,
                   const void* wo_att, void* out, void* qkv, void* ctx, float* lse, hipStream_t st) {
  const long long N = (long long)c.G * c.S;
  const int A = d.heads * d.d;
  int rc = dense_gemm(c, N, c.M, 3 * A, false, u, wqkv, qkv, st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_attention_core(c.act_dtype, qkv, ctx, lse, d.B, d.L, d.heads, d.d, st);
  if (rc != MOE_OK) return rc;
  return dense_gemm(c, N, A, c.M, false, ctx, wo_att, out, st);
}

// Training form of the pair: every sub-layer keeps what its derivative needs.
struct EncoderTrainWs { size_t n[4], a, b, c, sub, hden, qkv[2], ctx[2], lse[2], moe, total; };
EncoderTrainWs carve_enc_train(const moe_config& c, const moe_encoder_dims& d) {
  const size_t N = (size_t)c.G * c.S, A = (size_t)d.heads * d.d;
  const size_t elt = c.act_dtype == MOE_F32 ? 4 : 2;
  EncoderTrainWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  for (int i = 0; i < 4; ++i) w.n[i] = take(N * c.M * elt);
  w.a = take(N * c.M * elt);
  w.b = take(N * c.M * elt);
  w.c = take(N * c.M * elt);
  w.sub = take(N * c.M * elt);
  w.hden = take(N * c.H * elt);
  for (int i = 0; i < 2; ++i) {
    w.qkv[i] = take(N * 3 * A * elt);
    w.ctx[i] = take(N * A * elt);
    w.lse[i] = take((size_t)d.B * d.heads * d.L * sizeof(float));
  }
  w.moe = take(carve(c, true).total);
  w.total = off;
  return w;
}

struct EncoderBwdWs { size_t g[2], dn, dqkv, dctx, dhden, dvec, partial, wpart, moe, total; };
EncoderBwdWs carve_enc_bwd(const moe_config& c, const moe_encoder_dims& d) {
  const size_t N = (size_t)c.G * c.S, A = (size_t)d.heads * d.d;
  const size_t elt = c.act_dtype == MOE_F32 ? 4 : 2;
  EncoderBwdWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  w.g[0] = take(N * c.M * elt);
  w.g[1] = take(N * c.M * elt);
  w.dn = take(N * c.M * elt);
  w.dqkv = take(N * 3 * A * elt);
  w.dctx = take(N * A * elt);
  w.dhden = take(N * c.H * elt);
  w.dvec = take((size_t)d.B * d.heads * d.L * sizeof(float));
  w.partial = take((size_t)moe::layer_norm_bwd_parts((long long)N) * 2 * c.M * sizeof(float));
  // token ranges of the dense weight gradients (the largest of the four shapes)
  size_t wp = moe::dense_wgrad_partial_bytes(c.act_dtype, (long long)N, (int)A, c.M);
  const size_t wp2 = moe::dense_wgrad_partial_bytes(c.act_dtype, (long long)N, c.M, 3 * (int)A);
  const size_t wp3 = moe::dense_wgrad_partial_bytes(c.act_dtype, (long long)N, c.M, c.H);
  const size_t wp4 = moe::dense_wgrad_partial_bytes(c.act_dtype, (long long)N, c.H, c.M);
  wp = wp > wp2 ? wp : wp2;
  wp = wp > wp3 ? wp : wp3;
  wp = wp > wp4 ? wp : wp4;
  w.wpart = take(wp);
  w.moe = take(carve_bwd(c).total);
  w.total = off;
  return w;
}

// one-expert configuration for the dense layers' gradient GEMMs: rows tokens, widths in -> out
moe_config dense_cfg(const moe_config& c, long long rows, int in, int out) {
  moe_config g = c;
  g.E = 1;
  g.G = 1;
  g.C = (int)rows;
  g.M = in;
  g.H = out;
  return g;
}

// gradients of out = Attention(u): dout [N,M] -> du [N,M], dwqkv [M,3A], dwo_att [A,M]
int attention_bwd_impl(const moe_config& c, const moe_encoder_dims& d, const void* u,
                       const void* wqkv, const void* wo_att, const void* qkv, const void* ctx,
                       const float* lse, const void* dout, void* du, void* dwqkv, void* dwo_att,
                       void* dqkv, void* dctx, float* dvec, float* wpart, hipStream_t st) {
  const long long N = (long long)c.G * c.S;
  const int A = d.heads * d.d;
  // out = ctx . wo_att
  int rc = moe::launch_dense_wgrad(c, N, A, c.M, ctx, dout, dwo_att, wpart, st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_expert_dgrad1(dense_cfg(c, N, A, c.M), dout, wo_att, dctx, nullptr, st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_attention_core_bwd(c.act_dtype, qkv, ctx, dctx, lse, dqkv, dvec, d.B, d.L, d.heads,
                                      d.d, st);
  if (rc != MOE_OK) return rc;
  // qkv = u . wqkv
  rc = moe::launch_dense_wgrad(c, N, c.M, 3 * A, u, dqkv, dwqkv, wpart, st);
  if (rc != MOE_OK) return rc;
  return moe::launch_expert_dgrad1(dense_cfg(c, N, c.M, 3 * A), dqkv, wqkv, du, nullptr, st);
}

}  // namespace

extern "C" {

const char* moe_status_string(int status) {
  switch (status) {
    case MOE_OK: return "MOE_OK";
    case MOE_EINVAL: return "MOE_EINVAL: invalid argument";
    case MOE_EUNSUPPORTED: return "MOE_EUNSUPPORTED: shape not supported by the kernels";
    case MOE_EWORKSPACE: return "MOE_EWORKSPACE: workspace too small";
    case MOE_EHIP: return "MOE_EHIP: kernel launch failed";
    default: return "unknown moe_status";
  }
}

int moe_prepare(void) {
  int rc = moe::prepare_expert_gemm();
  if (rc == MOE_OK) rc = moe::prepare_gate();
  if (rc == MOE_OK) rc = moe::prepare_attention_bwd();
  void* p = nullptr;
  if (rc == MOE_OK) rc = gate_scratch_ptr(&p);
  return rc;
}

int moe_gate_workspace_bytes(const moe_config* cfg, size_t* bytes) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = moe::gate_workspace_bytes(*cfg);
  return MOE_OK;
}

int moe_workspace_bytes(const moe_config* cfg, size_t* bytes) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = carve(*cfg, false).total;
  return MOE_OK;
}

int moe_train_workspace_bytes(const moe_config* cfg, size_t* bytes) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = carve(*cfg, true).total;
  return MOE_OK;
}

int moe_forward_fuses_dispatch(const moe_config* cfg, int* fused) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (fused == nullptr) return MOE_EINVAL;
  *fused = moe::expert_gemm1_can_gather(*cfg) ? 1 : 0;
  return MOE_OK;
}

int moe_gate_pack_bytes(const moe_config* cfg, size_t* bytes) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = moe::gate_pack_bytes(*cfg);
  return MOE_OK;
}

int moe_gate_pack(const moe_config* cfg, const float* wg, void* wg_packed, void* stream) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (wg == nullptr || !aligned16(wg)) return MOE_EINVAL;
  if (moe::gate_pack_bytes(*cfg) == 0) return MOE_OK;
  if (wg_packed == nullptr || (reinterpret_cast<uintptr_t>(wg_packed) & 255u) != 0) return MOE_EINVAL;
  return moe::launch_gate_pack(*cfg, wg, wg_packed, static_cast<hipStream_t>(stream));
}

int moe_forward_prepacked(const moe_config* cfg, const void* x, const float* wg,
                          const void* wg_packed, const float* u, const void* wi, const void* wo,
                          void* y, float* aux, void* ws, size_t ws_bytes, void* stream,
                          void* const* events) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (moe::gate_pack_bytes(*cfg) == 0) wg_packed = nullptr;       // this gate reads wg itself
  else if (wg_packed == nullptr || (reinterpret_cast<uintptr_t>(wg_packed) & 255u) != 0)
    return MOE_EINVAL;
  return forward_impl(cfg, x, wg, u, wi, wo, y, aux, ws, ws_bytes, stream, events, false, wg_packed);
}

int moe_gate_prepacked(const moe_config* cfg, const void* x, const float* wg, const void* wg_packed,
                       const float* u, int32_t* expert_idx, int32_t* slot, float* weight,
                       int32_t* fill, int32_t* src_token, int32_t* c1, float* mean_gate,
                       float* aux, float* gates_opt, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {x, wg, u, expert_idx, slot, weight, fill, src_token, c1, mean_gate, aux, ws};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if (gates_opt != nullptr && !aligned16(gates_opt)) return MOE_EINVAL;
  if (moe::gate_pack_bytes(*cfg) == 0) wg_packed = nullptr;
  else if (wg_packed == nullptr || (reinterpret_cast<uintptr_t>(wg_packed) & 255u) != 0)
    return MOE_EINVAL;
  if (ws_bytes < moe::gate_workspace_bytes(*cfg)) return MOE_EWORKSPACE;
  return moe::launch_gate(*cfg, x, wg, u, expert_idx, slot, weight, fill, src_token, c1,
                          mean_gate, aux, gates_opt, ws, nullptr, nullptr, wg_packed,
                          static_cast<hipStream_t>(stream));
}

int moe_gate(const moe_config* cfg, const void* x, const float* wg, const float* u,
             int32_t* expert_idx, int32_t* slot, float* weight, int32_t* fill,
             int32_t* src_token, int32_t* c1, float* mean_gate, float* aux, float* gates_opt,
             void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {x, wg, u, expert_idx, slot, weight, fill, src_token, c1, mean_gate, aux, ws};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if (gates_opt != nullptr && !aligned16(gates_opt)) return MOE_EINVAL;
  if (ws_bytes < moe::gate_workspace_bytes(*cfg)) return MOE_EWORKSPACE;
  return moe::launch_gate(*cfg, x, wg, u, expert_idx, slot, weight, fill, src_token, c1,
                          mean_gate, aux, gates_opt, ws, nullptr, nullptr, nullptr,
                          static_cast<hipStream_t>(stream));
}

int moe_gate_noalloc_max_bytes(size_t* bytes) {
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = kGateScratchBytes;
  return MOE_OK;
}

int moe_gate_noalloc(const moe_config* cfg, const void* x, const float* wg, const float* u,
                     int32_t* expert_idx, int32_t* slot, float* weight, int32_t* fill,
                     int32_t* src_token, int32_t* c1, float* mean_gate, float* aux,
                     float* gates_opt, void* stream) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {x, wg, u, expert_idx, slot, weight, fill, src_token, c1, mean_gate, aux};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if (gates_opt != nullptr && !aligned16(gates_opt)) return MOE_EINVAL;
  if (moe::gate_workspace_bytes(*cfg) > kGateScratchBytes) return MOE_EWORKSPACE;
  void* ws = nullptr;
  const int rs = gate_scratch_ptr(&ws);
  if (rs != MOE_OK) return rs;
  // every word of the scratch that the kernels read is written earlier in the same call
  // (chunk histograms, gate sums and the packed weights), so nothing has to be cleared
  return moe::launch_gate(*cfg, x, wg, u, expert_idx, slot, weight, fill, src_token, c1,
                          mean_gate, aux, gates_opt, ws, nullptr, nullptr, nullptr,
                          static_cast<hipStream_t>(stream));
}

int moe_dispatch(const moe_config* cfg, const void* x, const int32_t* src_token, void* buf,
                 void* stream) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {x, src_token, buf};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  return moe::launch_dispatch(*cfg, x, src_token, buf, nullptr, static_cast<hipStream_t>(stream));
}

int moe_forward_packs_rows(const moe_config* cfg, int* packed) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (packed == nullptr) return MOE_EINVAL;
  *packed = moe::expert_ffn_can_pack(*cfg) ? 1 : 0;
  return MOE_OK;
}

int moe_expert_ffn_workspace_bytes(const moe_config* cfg, size_t* bytes) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  const size_t elt = cfg->act_dtype == MOE_F32 ? 4 : 2;
  *bytes = moe::expert_ffn_can_pack(*cfg)
               ? moe::row_packing_bytes(*cfg) + align_up((size_t)cfg->M * elt, 256) : 0;
  return MOE_OK;
}

int moe_expert_ffn(const moe_config* cfg, const void* buf, const int32_t* fill, const void* wi,
                   const void* wo, void* h_ws, void* out, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {buf, wi, wo, h_ws, out};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if (fill != nullptr && !aligned16(fill)) return MOE_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (fill != nullptr && ws != nullptr && moe::expert_ffn_can_pack(*cfg)) {
    // occupied rows only: row maps from fill, the first GEMM gathers the occupied rows of buf,
    // the second sends its rows back to their slots of out
    if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MOE_EINVAL;
    const size_t maps = moe::row_packing_bytes(*cfg);
    if (ws_bytes < maps + align_up((size_t)cfg->M * 2, 256)) return MOE_EWORKSPACE;
    const moe::RowPacking pk = moe::carve_row_packing(*cfg, ws);
    void* zero_row = static_cast<char*>(ws) + maps;
    int r = moe::launch_row_maps_from_fill(*cfg, fill, pk, zero_row, st);
    if (r != MOE_OK) return r;
    return moe::launch_expert_ffn_packed(*cfg, buf, pk, zero_row, wi, wo, h_ws, out, true, nullptr, st,
                                         nullptr);
  }
  const int rc1 = moe::launch_expert_gemm1(*cfg, buf, wi, h_ws, st);
  if (rc1 != MOE_OK) return rc1;
  return moe::launch_expert_gemm2(*cfg, h_ws, wo, out, st);
}

int moe_combine(const moe_config* cfg, const void* out, const int32_t* expert_idx,
                const int32_t* slot, const float* weight, void* y, void* stream) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {out, expert_idx, slot, weight, y};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  return moe::launch_combine(*cfg, out, expert_idx, slot, weight, nullptr, y,
                             static_cast<hipStream_t>(stream));
}

int moe_forward_events(const moe_config* cfg, const void* x, const float* wg, const float* u,
                       const void* wi, const void* wo, void* y, float* aux, void* ws,
                       size_t ws_bytes, void* stream, void* const* events) {
  return forward_impl(cfg, x, wg, u, wi, wo, y, aux, ws, ws_bytes, stream, events, false);
}

int moe_forward_train(const moe_config* cfg, const void* x, const float* wg, const float* u,
                      const void* wi, const void* wo, void* y, float* aux, void* ws,
                      size_t ws_bytes, void* stream) {
  return forward_impl(cfg, x, wg, u, wi, wo, y, aux, ws, ws_bytes, stream, nullptr, true);
}

int moe_backward_workspace_bytes(const moe_config* cfg, size_t* bytes) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = carve_bwd(*cfg).total;
  return MOE_OK;
}

int moe_backward_events(const moe_config* cfg, const void* x, const float* wg, const void* wi,
                        const void* wo, const void* dy, const float* daux, const void* fwd_ws,
                        size_t fwd_ws_bytes, void* dx, float* dwg, void* dwi, void* dwo, void* ws,
                        size_t ws_bytes, void* stream, void* const* events) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {x, wg, wi, wo, dy, daux, fwd_ws, dx, dwg, dwi, dwo, ws};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MOE_EINVAL;
  if ((reinterpret_cast<uintptr_t>(fwd_ws) & 255u) != 0) return MOE_EINVAL;
  if (events != nullptr)
    for (int i = 0; i < MOE_BACKWARD_EVENTS; ++i)
      if (events[i] == nullptr) return MOE_EINVAL;
  const ForwardWs f = carve(*cfg, true);
  const BackwardWs b = carve_bwd(*cfg);
  if (fwd_ws_bytes < f.total || ws_bytes < b.total) return MOE_EWORKSPACE;
  const char* fb = static_cast<const char*>(fwd_ws);
  char* base = static_cast<char*>(ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  auto mark = [&](int i) {
    return events == nullptr ||
           hipEventRecord(static_cast<hipEvent_t>(events[i]), st) == hipSuccess;
  };
  const int32_t* expert_idx = reinterpret_cast<const int32_t*>(fb + f.expert_idx);
  const int32_t* slot = reinterpret_cast<const int32_t*>(fb + f.slot);
  const float* weight = reinterpret_cast<const float*>(fb + f.weight);
  const int32_t* src_token = reinterpret_cast<const int32_t*>(fb + f.src_token);
  float* dweight = reinterpret_cast<float*>(base + b.dweight);
  const moe::GateBwdWs gw{reinterpret_cast<float*>(base + b.dz),
                          reinterpret_cast<moe::bf16_t*>(base + b.dzp),
                          reinterpret_cast<moe::bf16_t*>(base + b.wgp),
                          reinterpret_cast<float*>(base + b.dxg),
                          reinterpret_cast<float*>(base + b.dwg_partial)};
  // the training forward packed the occupied rows of each expert when the shape allows it:
  // h, out and the row maps in its workspace are in that layout, and so are dout, dh, dbuf, buf
  const bool packed = moe::expert_ffn_can_pack(*cfg);
  const moe::RowPacking pk = moe::carve_row_packing(*cfg, const_cast<char*>(fb) + f.packing);
  const int32_t* kept = packed ? pk.kept : nullptr;
  const int32_t* rows_src = packed ? pk.packed_src : src_token;
  if (!mark(0)) return MOE_EHIP;
  rc = moe::launch_combine_bwd(*cfg, dy, fb + f.out, rows_src, expert_idx, weight, base + b.dout,
                               dweight, kept, st);
  if (rc != MOE_OK) return rc;
  if (!mark(1)) return MOE_EHIP;
  rc = moe::launch_expert_dgrad2(*cfg, base + b.dout, wo, fb + f.h,
                                 moe::expert_gemm1_can_gather(*cfg) ? fb + f.signbits : nullptr,
                                 base + b.dh, kept, st);
  if (rc != MOE_OK) return rc;
  if (!mark(2)) return MOE_EHIP;
  rc = moe::launch_expert_wgrad2(*cfg, fb + f.h, base + b.dout, dwo, kept, st);
  if (rc != MOE_OK) return rc;
  if (!mark(3)) return MOE_EHIP;
  rc = moe::launch_expert_dgrad1(*cfg, base + b.dh, wi, base + b.dbuf, kept, st);
  if (rc != MOE_OK) return rc;
  if (!mark(4)) return MOE_EHIP;
  rc = moe::launch_dispatch(*cfg, x, rows_src, base + b.buf, kept, st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_expert_wgrad1(*cfg, base + b.buf, base + b.dh, dwi, kept, st);
  if (rc != MOE_OK) return rc;
  if (!mark(5)) return MOE_EHIP;
  rc = moe::launch_gate_bwd(*cfg, x, wg, reinterpret_cast<const float*>(fb + f.gates), expert_idx,
                            slot, dweight, reinterpret_cast<const int32_t*>(fb + f.c1), daux, gw,
                            dwg, st);
  if (rc != MOE_OK) return rc;
  if (!mark(6)) return MOE_EHIP;
  rc = moe::launch_dx(*cfg, wg, base + b.dbuf, expert_idx, slot, gw, dx,
                      packed ? pk.row_base : nullptr, st);
  if (rc != MOE_OK) return rc;
  return mark(7) ? MOE_OK : MOE_EHIP;
}

int moe_backward(const moe_config* cfg, const void* x, const float* wg, const void* wi,
                 const void* wo, const void* dy, const float* daux, const void* fwd_ws,
                 size_t fwd_ws_bytes, void* dx, float* dwg, void* dwi, void* dwo, void* ws,
                 size_t ws_bytes, void* stream) {
  return moe_backward_events(cfg, x, wg, wi, wo, dy, daux, fwd_ws, fwd_ws_bytes, dx, dwg, dwi, dwo,
                             ws, ws_bytes, stream, nullptr);
}

int moe_forward(const moe_config* cfg, const void* x, const float* wg, const float* u,
                const void* wi, const void* wo, void* y, float* aux, void* ws, size_t ws_bytes,
                void* stream) {
  return moe_forward_events(cfg, x, wg, u, wi, wo, y, aux, ws, ws_bytes, stream, nullptr);
}

int moe_add_layer_norm(const moe_config* cfg, const void* x, const void* delta, const float* gamma,
                       const float* beta, void* sum_out, void* norm_out, void* stream) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {x, gamma, beta, norm_out};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if (delta != nullptr && (sum_out == nullptr || !aligned16(delta) || !aligned16(sum_out)))
    return MOE_EINVAL;
  return moe::launch_add_layer_norm(cfg->act_dtype, x, delta, gamma, beta, sum_out, norm_out,
                                    (long long)cfg->G * cfg->S, cfg->M,
                                    static_cast<hipStream_t>(stream));
}

int moe_attention_workspace_bytes(const moe_config* cfg, const moe_encoder_dims* dims, size_t* bytes) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if ((rc = check_dims(cfg, dims)) != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = carve_att(*cfg, *dims).total;
  return MOE_OK;
}

int moe_encoder_workspace_bytes(const moe_config* cfg, const moe_encoder_dims* dims, size_t* bytes) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if ((rc = check_dims(cfg, dims)) != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = carve_enc(*cfg, *dims).total;
  return MOE_OK;
}

int moe_self_attention(const moe_config* cfg, const moe_encoder_dims* dims, const void* u,
                       const void* wqkv, const void* wo_att, void* out, void* ws, size_t ws_bytes,
                       void* stream) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if ((rc = check_dims(cfg, dims)) != MOE_OK) return rc;
  const void* req[] = {u, wqkv, wo_att, out, ws};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MOE_EINVAL;
  if (ws_bytes < carve_att(*cfg, *dims).total) return MOE_EWORKSPACE;
  const AttentionWs aw = carve_att(*cfg, *dims);
  return attention_impl(*cfg, *dims, u, wqkv, wo_att, out, static_cast<char*>(ws) + aw.qkv,
                        static_cast<char*>(ws) + aw.ctx, nullptr, static_cast<hipStream_t>(stream));
}

int moe_dense_ffn(const moe_config* cfg, const void* u, const void* w1, const void* w2, void* h_ws,
                  void* out, void* stream) {
  const int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  const void* req[] = {u, w1, w2, h_ws, out};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long long N = (long long)cfg->G * cfg->S;
  const int rc1 = dense_gemm(*cfg, N, cfg->M, cfg->H, true, u, w1, h_ws, st);
  if (rc1 != MOE_OK) return rc1;
  return dense_gemm(*cfg, N, cfg->H, cfg->M, false, h_ws, w2, out, st);
}

int moe_encoder_pair_forward(const moe_config* cfg, const moe_encoder_dims* dims, const void* x,
                             const moe_encoder_weights* w, const float* u, void* y, float* aux,
                             void* ws, size_t ws_bytes, void* stream) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if ((rc = check_dims(cfg, dims)) != MOE_OK) return rc;
  if (w == nullptr) return MOE_EINVAL;
  const void* req[] = {x, u, y, aux, ws, w->wqkv[0], w->wqkv[1], w->wo_att[0], w->wo_att[1], w->w1,
                       w->w2, w->wg, w->wi, w->wo, w->ln_gamma[0], w->ln_gamma[1], w->ln_gamma[2],
                       w->ln_gamma[3], w->ln_beta[0], w->ln_beta[1], w->ln_beta[2], w->ln_beta[3]};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MOE_EINVAL;
  const EncoderWs e = carve_enc(*cfg, *dims);
  if (ws_bytes < e.total) return MOE_EWORKSPACE;
  char* base = static_cast<char*>(ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long long N = (long long)cfg->G * cfg->S;
  const int dt = cfg->act_dtype;
  void *norm = base + e.norm, *sub = base + e.sub, *a = base + e.a, *b = base + e.b, *c = base + e.c;
  // layer 1: a = x + Attention_1(LN_1(x)); b = a + FFN(LN_2(a))
  rc = moe::launch_add_layer_norm(dt, x, nullptr, w->ln_gamma[0], w->ln_beta[0], nullptr, norm, N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  const AttentionWs aw = carve_att(*cfg, *dims);
  rc = attention_impl(*cfg, *dims, norm, w->wqkv[0], w->wo_att[0], sub, base + e.att + aw.qkv,
                      base + e.att + aw.ctx, nullptr, st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_add_layer_norm(dt, x, sub, w->ln_gamma[1], w->ln_beta[1], a, norm, N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  rc = dense_gemm(*cfg, N, cfg->M, cfg->H, true, norm, w->w1, base + e.hden, st);
  if (rc != MOE_OK) return rc;
  rc = dense_gemm(*cfg, N, cfg->H, cfg->M, false, base + e.hden, w->w2, sub, st);
  if (rc != MOE_OK) return rc;
  // layer 2: c = b + Attention_2(LN_3(b)); y = c + MoE(LN_4(c))
  rc = moe::launch_add_layer_norm(dt, a, sub, w->ln_gamma[2], w->ln_beta[2], b, norm, N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  rc = attention_impl(*cfg, *dims, norm, w->wqkv[1], w->wo_att[1], sub, base + e.att + aw.qkv,
                      base + e.att + aw.ctx, nullptr, st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_add_layer_norm(dt, b, sub, w->ln_gamma[3], w->ln_beta[3], c, norm, N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  rc = forward_impl(cfg, norm, w->wg, u, w->wi, w->wo, sub, aux, base + e.moe, carve(*cfg, false).total,
                    stream, nullptr, false);
  if (rc != MOE_OK) return rc;
  return moe::launch_add_rows(dt, c, sub, y, N * cfg->M, st);
}

int moe_encoder_train_workspace_bytes(const moe_config* cfg, const moe_encoder_dims* dims, size_t* bytes) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if ((rc = check_dims(cfg, dims)) != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = carve_enc_train(*cfg, *dims).total;
  return MOE_OK;
}

int moe_encoder_backward_workspace_bytes(const moe_config* cfg, const moe_encoder_dims* dims,
                                         size_t* bytes) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if ((rc = check_dims(cfg, dims)) != MOE_OK) return rc;
  if (bytes == nullptr) return MOE_EINVAL;
  *bytes = carve_enc_bwd(*cfg, *dims).total;
  return MOE_OK;
}

int moe_encoder_pair_forward_train(const moe_config* cfg, const moe_encoder_dims* dims, const void* x,
                                   const moe_encoder_weights* w, const float* u, void* y, float* aux,
                                   void* ws, size_t ws_bytes, void* stream) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if ((rc = check_dims(cfg, dims)) != MOE_OK) return rc;
  if (w == nullptr) return MOE_EINVAL;
  const void* req[] = {x, u, y, aux, ws, w->wqkv[0], w->wqkv[1], w->wo_att[0], w->wo_att[1], w->w1,
                       w->w2, w->wg, w->wi, w->wo, w->ln_gamma[0], w->ln_gamma[1], w->ln_gamma[2],
                       w->ln_gamma[3], w->ln_beta[0], w->ln_beta[1], w->ln_beta[2], w->ln_beta[3]};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MOE_EINVAL;
  const EncoderTrainWs e = carve_enc_train(*cfg, *dims);
  if (ws_bytes < e.total) return MOE_EWORKSPACE;
  char* base = static_cast<char*>(ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long long N = (long long)cfg->G * cfg->S;
  const int dt = cfg->act_dtype;
  void *sub = base + e.sub, *a = base + e.a, *b = base + e.b, *c = base + e.c;
  auto lse = [&](int i) { return reinterpret_cast<float*>(base + e.lse[i]); };
  rc = moe::launch_add_layer_norm(dt, x, nullptr, w->ln_gamma[0], w->ln_beta[0], nullptr, base + e.n[0], N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  rc = attention_impl(*cfg, *dims, base + e.n[0], w->wqkv[0], w->wo_att[0], sub, base + e.qkv[0],
                      base + e.ctx[0], lse(0), st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_add_layer_norm(dt, x, sub, w->ln_gamma[1], w->ln_beta[1], a, base + e.n[1], N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  rc = dense_gemm(*cfg, N, cfg->M, cfg->H, true, base + e.n[1], w->w1, base + e.hden, st);
  if (rc != MOE_OK) return rc;
  rc = dense_gemm(*cfg, N, cfg->H, cfg->M, false, base + e.hden, w->w2, sub, st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_add_layer_norm(dt, a, sub, w->ln_gamma[2], w->ln_beta[2], b, base + e.n[2], N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  rc = attention_impl(*cfg, *dims, base + e.n[2], w->wqkv[1], w->wo_att[1], sub, base + e.qkv[1],
                      base + e.ctx[1], lse(1), st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_add_layer_norm(dt, b, sub, w->ln_gamma[3], w->ln_beta[3], c, base + e.n[3], N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  rc = forward_impl(cfg, base + e.n[3], w->wg, u, w->wi, w->wo, sub, aux, base + e.moe,
                    carve(*cfg, true).total, stream, nullptr, true);
  if (rc != MOE_OK) return rc;
  return moe::launch_add_rows(dt, c, sub, y, N * cfg->M, st);
}

int moe_encoder_pair_backward(const moe_config* cfg, const moe_encoder_dims* dims, const void* x,
                              const moe_encoder_weights* w, const void* dy, const float* daux,
                              const void* fwd_ws, size_t fwd_ws_bytes, void* dx,
                              const moe_encoder_grads* g, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_config(cfg);
  if (rc != MOE_OK) return rc;
  if ((rc = check_dims(cfg, dims)) != MOE_OK) return rc;
  if (w == nullptr || g == nullptr) return MOE_EINVAL;
  const void* req[] = {x, dy, daux, fwd_ws, dx, ws, w->wqkv[0], w->wqkv[1], w->wo_att[0], w->wo_att[1],
                       w->w1, w->w2, w->wg, w->wi, w->wo, w->ln_gamma[0], w->ln_gamma[1],
                       w->ln_gamma[2], w->ln_gamma[3], g->wqkv[0], g->wqkv[1], g->wo_att[0],
                       g->wo_att[1], g->w1, g->w2, g->wg, g->wi, g->wo, g->ln_gamma[0], g->ln_gamma[1],
                       g->ln_gamma[2], g->ln_gamma[3], g->ln_beta[0], g->ln_beta[1], g->ln_beta[2],
                       g->ln_beta[3]};
  for (const void* p : req)
    if (p == nullptr || !aligned16(p)) return MOE_EINVAL;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MOE_EINVAL;
  if ((reinterpret_cast<uintptr_t>(fwd_ws) & 255u) != 0) return MOE_EINVAL;
  const EncoderTrainWs e = carve_enc_train(*cfg, *dims);
  const EncoderBwdWs bw = carve_enc_bwd(*cfg, *dims);
  if (fwd_ws_bytes < e.total || ws_bytes < bw.total) return MOE_EWORKSPACE;
  const char* f = static_cast<const char*>(fwd_ws);
  char* base = static_cast<char*>(ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long long N = (long long)cfg->G * cfg->S;
  const int dt = cfg->act_dtype;
  void *g0 = base + bw.g[0], *g1 = base + bw.g[1], *dn = base + bw.dn;
  float* partial = reinterpret_cast<float*>(base + bw.partial);
  float* dvec = reinterpret_cast<float*>(base + bw.dvec);
  float* wpart = reinterpret_cast<float*>(base + bw.wpart);
  auto lse = [&](int i) { return reinterpret_cast<const float*>(f + e.lse[i]); };

  // y = c + MoE(n4): the MoE layer's gradients; dn = d L / d n4
  rc = moe_backward(cfg, f + e.n[3], w->wg, w->wi, w->wo, dy, daux, f + e.moe, carve(*cfg, true).total, dn,
                    g->wg, g->wi, g->wo, base + bw.moe, carve_bwd(*cfg).total, stream);
  if (rc != MOE_OK) return rc;
  // g0 = d L / d c = dy + LN4'(dn)
  rc = moe::launch_layer_norm_bwd(dt, f + e.c, dn, w->ln_gamma[3], dy, g0, partial, g->ln_gamma[3],
                                  g->ln_beta[3], N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  // c = b + Attention_2(n3)
  rc = attention_bwd_impl(*cfg, *dims, f + e.n[2], w->wqkv[1], w->wo_att[1], f + e.qkv[1],
                          f + e.ctx[1], lse(1), g0, dn, g->wqkv[1], g->wo_att[1], base + bw.dqkv,
                          base + bw.dctx, dvec, wpart, st);
  if (rc != MOE_OK) return rc;
  rc = moe::launch_layer_norm_bwd(dt, f + e.b, dn, w->ln_gamma[2], g0, g1, partial, g->ln_gamma[2],
                                  g->ln_beta[2], N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  // b = a + relu(n2 w1) w2
  {
    const moe_config fc = dense_cfg(*cfg, N, cfg->M, cfg->H);
    rc = moe::launch_dense_wgrad(*cfg, N, cfg->H, cfg->M, f + e.hden, g1, g->w2, wpart, st);
    if (rc != MOE_OK) return rc;
    rc = moe::launch_expert_dgrad2(fc, g1, w->w2, f + e.hden, nullptr, base + bw.dhden, nullptr, st);
    if (rc != MOE_OK) return rc;
    rc = moe::launch_dense_wgrad(*cfg, N, cfg->M, cfg->H, f + e.n[1], base + bw.dhden, g->w1, wpart, st);
    if (rc != MOE_OK) return rc;
    rc = moe::launch_expert_dgrad1(fc, base + bw.dhden, w->w1, dn, nullptr, st);
    if (rc != MOE_OK) return rc;
  }
  rc = moe::launch_layer_norm_bwd(dt, f + e.a, dn, w->ln_gamma[1], g1, g0, partial, g->ln_gamma[1],
                                  g->ln_beta[1], N, cfg->M, st);
  if (rc != MOE_OK) return rc;
  // a = x + Attention_1(n1)
  rc = attention_bwd_impl(*cfg, *dims, f + e.n[0], w->wqkv[0], w->wo_att[0], f + e.qkv[0],
                          f + e.ctx[0], lse(0), g0, dn, g->wqkv[0], g->wo_att[0], base + bw.dqkv,
                          base + bw.dctx, dvec, wpart, st);
  if (rc != MOE_OK) return rc;
  return moe::launch_layer_norm_bwd(dt, x, dn, w->ln_gamma[0], g0, dx, partial, g->ln_gamma[0],
                                    g->ln_beta[0], N, cfg->M, st);
}

}  // extern "C"
