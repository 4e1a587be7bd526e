// C ABI of the scoring library: argument validation, workspace carving and the
// launch sequence of the hot path.  See include/mrl.h for the contract.
#include "../../include/mrl.h"
#include "../../include/mrl_diag.h"
#include "mrl_internal.h"

#include <cstring>
#include <mutex>
#include <vector>

// Scratch space of mrl_token_logprobs_static.  In host code the array's name is only a handle
// for the symbol lookup in static_scratch_ptr(), never a device address: every device holds its
// own copy at its own address, looked up once per device with that device current.
static __device__ __align__(256) unsigned char scratch[MRL_STATIC_SCRATCH_BYTES];

namespace mrl {
namespace {

constexpr int kDefaultChunkBf16 = 65536;   // rows per pass: amortises the fp32 dW read-modify-write (20 GB of stash at V = 151936)
constexpr int kFwdSubChunk = 16384;        // forward launches cover this many rows: their H rows stay in the Infinity Cache
constexpr int kDefaultChunkF32 = 2048;
constexpr int64_t kMaxSlots = (int64_t)1 << 30;

// ------------------------------------------------------------------ profiling
struct ProfRec { int cls; hipEvent_t start, stop; };
std::mutex g_prof_mu;
std::atomic<bool> g_prof_on{false};
std::vector<ProfRec> g_prof_log;
std::vector<hipEvent_t> g_event_pool;

hipEvent_t take_event() {
  if (!g_event_pool.empty()) { hipEvent_t e = g_event_pool.back(); g_event_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

}  // namespace

void prof_begin(int cls, hipStream_t stream) {
  if (!g_prof_on.load(std::memory_order_relaxed)) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  ProfRec r{cls, take_event(), take_event()};
  (void)hipEventRecord(r.start, stream);
  g_prof_log.push_back(r);
}
void prof_end(int cls, hipStream_t stream) {
  if (!g_prof_on.load(std::memory_order_relaxed)) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  for (size_t i = g_prof_log.size(); i-- > 0;)
    if (g_prof_log[i].cls == cls) { (void)hipEventRecord(g_prof_log[i].stop, stream); break; }
}

namespace {

struct Scope {
  int cls; hipStream_t s;
  Scope(int c, hipStream_t st) : cls(c), s(st) { prof_begin(cls, s); }
  ~Scope() { prof_end(cls, s); }
};

// ------------------------------------------------------------------ device check
int check_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) { (void)hipGetLastError(); return MRL_ERR_DEVICE; }
  static std::mutex mu;
  static std::vector<int> cache;   // 0 unknown, 1 ok, 2 unsupported
  std::lock_guard<std::mutex> lk(mu);
  if ((int)cache.size() <= dev) cache.resize(dev + 1, 0);
  if (cache[dev] == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return MRL_ERR_DEVICE; }
    cache[dev] = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
  }
  return cache[dev] == 1 ? MRL_OK : MRL_ERR_UNSUPPORTED_ARCH;
}

}  // namespace
int require_gfx950() { return check_device(); }
namespace {

// ------------------------------------------------------------------ built-in scratch buffer
// Device address of the current device's copy of `scratch`, or nullptr on failure.
void* static_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) { (void)hipGetLastError(); return nullptr; }
  static std::mutex mu;
  static std::vector<void*> per_device;
  std::lock_guard<std::mutex> lk(mu);
  if ((int)per_device.size() <= dev) per_device.resize(dev + 1, nullptr);
  if (per_device[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(::scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    per_device[dev] = ptr;
  }
  return per_device[dev];
}

// ------------------------------------------------------------------ workspace layout
struct Layout {
  size_t total = 0;
  size_t counters, row_index, block_counts, zt, part_max, part_sum, part_ez;
  size_t seq_len, seq_coef, seq_expo, group_count, lse_c, g_c, row_scale, loss_partials, Z, Pt, Ht, Wt;
  size_t dw_tail = 0;          // bf16: partial tiles of the dW launch's K-split tail
  size_t Hc = 0, Wp = 0;       // bf16: the pass's token rows, gathered and zero-padded to dp columns; W padded likewise (only if dp != d)
  int dp = 0;                  // bf16: d rounded up to the 128-wide panel pairs of the GEMM kernels
  int64_t ldh = 0;             // row stride of Hc and Wp
  int chunk_rows = 0, n_partials = 0;
  int64_t n_chunks = 0, Vp = 0, ldz = 0, ldr = 0;   // ldz: row stride of the stash (Z) and Wt, ldr: of Ht (and the fp32 path's Pt)
  int64_t epi_blocks_total = 0;
};

size_t take(size_t& off, size_t bytes) {
  const size_t at = off;
  off += (bytes + 255) / 256 * 256;
  return at;
}

Layout make_layout(int64_t N, int64_t B, int d, int V, int dtype, int chunk_rows, bool loss,
                   bool entropy = false) {
  Layout L;
  const bool bf16 = dtype == MRL_BF16;
  const size_t es = bf16 ? 2 : 4;
  L.chunk_rows = chunk_rows;
  L.n_chunks = N > 0 ? (N + chunk_rows - 1) / chunk_rows : 0;
  L.Vp = bf16 ? round_up(V, kTile) : V;
  // bf16 path: strides are padded by 64 elements (128 B) so that consecutive rows of a tile do
  // not fall onto the same L2 channel (a power-of-two row stride serialises the panel loads)
  L.ldz = bf16 ? L.Vp + 64 : L.Vp;
  L.ldr = bf16 ? chunk_rows + 64 : chunk_rows;
  L.n_partials = bf16 ? fwd_partials_bf16(V) : 1;
  L.epi_blocks_total = L.n_chunks * row_epilogue_blocks(chunk_rows);
  const int64_t nb = (N + 1023) / 1024;
  size_t off = 0;
  L.counters = take(off, 256);
  L.row_index = take(off, (size_t)(N + 1) * 4);
  L.block_counts = take(off, (size_t)(round_up(2 * nb, 2) * 4 + nb * 8 + 16));
  L.zt = take(off, (size_t)(N + 1) * 4);
  L.part_max = bf16 ? 0 : take(off, (size_t)L.n_partials * chunk_rows * 4);   // fp32 path only
  L.part_sum = take(off, (size_t)L.n_partials * chunk_rows * 4);
  L.part_ez = entropy ? take(off, (size_t)L.n_partials * chunk_rows * 4) : 0;
  const int dk = bf16 ? (int)round_up(d, 128) : d;   // rows of Ht / Wt
  if (bf16) {
    L.dp = dk;
    L.ldh = L.dp + 64;
    L.Hc = take(off, (size_t)chunk_rows * L.ldh * 2);
    if (L.dp != d) L.Wp = take(off, (size_t)V * L.ldh * 2);
  }
  if (loss) {
    L.seq_len = take(off, (size_t)(B + 1) * 4);
    L.seq_coef = take(off, (size_t)(B + 1) * 4);
    L.seq_expo = take(off, (size_t)(B + 1) * 4);
    L.group_count = take(off, (size_t)(B + 1) * 4);
    L.lse_c = take(off, (size_t)(N + 1) * 4);
    L.g_c = take(off, (size_t)(N + 1) * 4);
    L.row_scale = bf16 ? take(off, (size_t)(N + 1) * 4) : 0;
    L.loss_partials = take(off, (size_t)(L.epi_blocks_total + 1) * 10 * 8);
    L.Z = take(off, (size_t)chunk_rows * L.ldz * es);
    L.Pt = bf16 ? 0 : take(off, (size_t)L.Vp * L.ldr * es);   // fp32 path only: the bf16 dW GEMM reads P itself
    L.Ht = take(off, (size_t)dk * L.ldr * es);
    L.Wt = take(off, (size_t)dk * L.ldz * es);
    if (bf16) L.dw_tail = take(off, gemm_dw_tail_bytes());
  } else if (!bf16) {
    L.Z = take(off, (size_t)chunk_rows * L.ldz * es);
  }
  L.total = off;
  return L;
}

int default_chunk(int64_t N, int dtype) {
  const int cap = dtype == MRL_BF16 ? kDefaultChunkBf16 : kDefaultChunkF32;
  const int64_t need = round_up(N > 0 ? N : 1, kTile);
  return (int)(need < cap ? need : cap);
}

int check_common(int64_t N, int d, int V, int dtype) {
  if (dtype != MRL_F32 && dtype != MRL_BF16) return MRL_ERR_DTYPE;
  if (N < 0 || N > kMaxSlots || d <= 0 || V <= 0) return MRL_ERR_SHAPE;
  if (dtype == MRL_BF16 && d % 8 != 0) return MRL_ERR_SHAPE;   // 16-byte rows
  if ((int64_t)V > ((int64_t)1 << 24) || d > (1 << 20)) return MRL_ERR_SHAPE;
  return MRL_OK;
}

int check_cfg(const mrl_loss_config* c) {
  if (!(c->clip_eps_low >= 0.f) || !(c->clip_eps_high >= 0.f) || !(c->clip_eps_low <= 1.f)) return MRL_ERR_CONFIG;
  if (!(c->kl_beta >= 0.f) || !(c->sgt_lambda >= 0.f)) return MRL_ERR_CONFIG;
  if (c->loss_agg != 0 && c->loss_agg != 1) return MRL_ERR_CONFIG;
  if (c->accumulate_dw != 0 && c->accumulate_dw != 1) return MRL_ERR_CONFIG;
  if (c->dh_dtype != MRL_F32 && c->dh_dtype != MRL_BF16) return MRL_ERR_CONFIG;
  if (c->chunk_rows < 0 || c->chunk_rows % kTile != 0 || c->chunk_rows > (1 << 20)) return MRL_ERR_CONFIG;
  if (c->scored_rows_hint < 0) return MRL_ERR_CONFIG;
  if (c->ratio_level < 0 || c->ratio_level > 2) return MRL_ERR_CONFIG;
  if (c->debug_sync != 0 && c->debug_sync != 1) return MRL_ERR_CONFIG;
  if (c->ratio_level != 0 && c->loss_agg != 0) return MRL_ERR_CONFIG;
  return MRL_OK;
}

// pick the chunk size: the configured one, or the largest default-capped multiple of
// 256 whose layout fits into the caller's workspace
int pick_chunk(int64_t N, int64_t B, int d, int V, int dtype, int cfg_chunk, bool loss,
               size_t workspace_bytes, Layout& L, bool entropy = false) {
  if (cfg_chunk > 0) {
    L = make_layout(N, B, d, V, dtype, cfg_chunk, loss, entropy);
    return L.total <= workspace_bytes ? MRL_OK : MRL_ERR_WORKSPACE;
  }
  for (int r = default_chunk(N, dtype); r >= kTile; r = (r / 2) / kTile * kTile) {
    L = make_layout(N, B, d, V, dtype, r, loss, entropy);
    if (L.total <= workspace_bytes) return MRL_OK;
    if (r == kTile) break;
  }
  return MRL_ERR_WORKSPACE;
}

template <typename T>
T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<unsigned char*>(ws) + off); }

int last_error() {
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? MRL_OK : MRL_ERR_DEVICE;
}

// forward of one chunk: logits tile GEMM with fused (or, in fp32, separate) log-sum-exp
void forward_chunk(const void* H, const void* W, int d, int V, bool bf16, const Layout& L, void* ws,
                   int64_t c0, bool stash, hipStream_t s, bool entropy = false) {
  const int32_t* row_index = at<int32_t>(ws, L.row_index);
  const int64_t* n_scored = at<int64_t>(ws, L.counters);
  if (bf16) {
    {
      Scope sc(MRL_PROF_CONVERT, s);
      launch_gather_rows_b16(H, d, row_index + c0, at<void>(ws, L.Hc), L.ldh, 0, n_scored, c0, L.chunk_rows, d, L.dp, s);
    }
    const void* Wk = L.dp != d ? at<void>(ws, L.Wp) : W;
    const int64_t ldw = L.dp != d ? L.ldh : d;
    for (int sub = 0; sub < L.chunk_rows; sub += kFwdSubChunk) {
      const int rows = L.chunk_rows - sub < kFwdSubChunk ? L.chunk_rows - sub : kFwdSubChunk;
      Scope sc(MRL_PROF_GEMM_FWD, s);   // one event pair per kernel launch
      launch_gemm_fwd_bf16(Wk, ldw, at<uint16_t>(ws, L.Hc) + (size_t)sub * L.ldh, L.ldh, L.dp, at<float>(ws, L.zt),
                           n_scored, c0 + sub, rows, V, d,
                           at<float>(ws, L.part_sum) + sub, entropy ? at<float>(ws, L.part_ez) + sub : nullptr,
                           L.chunk_rows,
                           stash ? at<uint16_t>(ws, L.Z) + (size_t)sub * L.ldz : nullptr, L.ldz, s);
    }
  } else {
    Scope sc(MRL_PROF_GEMM_FWD, s);
    GemmF32Args g = {};
    g.A = static_cast<const float*>(H); g.lda = d; g.a_rows = row_index + c0;
    g.B = static_cast<const float*>(W); g.ldb = d;
    g.C = at<float>(ws, L.Z); g.ldc = L.ldz; g.c_rows = nullptr;
    g.M = L.chunk_rows; g.N = V; g.K = d;
    g.n_scored = n_scored; g.chunk_start = c0; g.chunk_rows = L.chunk_rows;
    g.m_dynamic = 1; g.k_dynamic = 0; g.accumulate = 0;
    launch_gemm_f32(g, s);
    launch_row_lse_f32(at<float>(ws, L.Z), L.ldz, n_scored, c0, L.chunk_rows, V, at<float>(ws, L.part_max),
                       at<float>(ws, L.part_sum), entropy ? at<float>(ws, L.part_ez) : nullptr, s);
  }
}

}  // namespace
}  // namespace mrl

using namespace mrl;

extern "C" {

const char* mrl_status_string(int status) {
  switch (status) {
    case MRL_OK: return "ok";
    case MRL_ERR_NULL: return "a required pointer is NULL";
    case MRL_ERR_SHAPE: return "invalid shape (sizes must be positive; bf16 needs d % 8 == 0)";
    case MRL_ERR_DTYPE: return "unknown dtype";
    case MRL_ERR_TARGET_RANGE: return "target id out of range";
    case MRL_ERR_GROUP_RANGE: return "group id out of range";
    case MRL_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MRL_ERR_CONFIG: return "invalid configuration value";
    case MRL_ERR_DEVICE: return "no usable HIP device or a HIP call failed";
    case MRL_ERR_UNSUPPORTED_ARCH: return "device is not gfx950 (no fallback path)";
    case MRL_ERR_SCRATCH_LIMIT: return "input too large for the library's built-in scratch buffer (use the workspace variant)";
    default: return "unknown status";
  }
}

int mrl_version(void) { return 100; }

int mrl_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on.store(on != 0);
  return MRL_OK;
}

int mrl_profile_collect(double* ms_per_class, int64_t* launches_per_class) {
  if (ms_per_class == nullptr || launches_per_class == nullptr) return MRL_ERR_NULL;
  for (int i = 0; i < MRL_PROF_NCLASS; ++i) { ms_per_class[i] = 0.0; launches_per_class[i] = 0; }
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (g_prof_log.empty()) return MRL_OK;
  if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); return MRL_ERR_DEVICE; }
  for (const ProfRec& r : g_prof_log) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess && r.cls >= 0 && r.cls < MRL_PROF_NCLASS) {
      ms_per_class[r.cls] += ms;
      launches_per_class[r.cls] += 1;
    } else {
      (void)hipGetLastError();
    }
    g_event_pool.push_back(r.start);
    g_event_pool.push_back(r.stop);
  }
  g_prof_log.clear();
  return MRL_OK;
}

// --------------------------------------------------------------------------- (1)
size_t mrl_token_logprobs_workspace(int64_t N, int32_t d, int32_t V, int32_t dtype) {
  if (check_common(N, d, V, dtype) != MRL_OK) return 0;
  return make_layout(N, 0, d, V, dtype, default_chunk(N, dtype), false).total;
}

size_t mrl_token_scores_workspace(int64_t N, int32_t d, int32_t V, int32_t dtype) {
  if (check_common(N, d, V, dtype) != MRL_OK) return 0;
  return make_layout(N, 0, d, V, dtype, default_chunk(N, dtype), false, true).total;
}

int mrl_token_scores(const void* hidden, const void* lm_head_w, const int32_t* target_ids,
                     const uint8_t* token_mask, int64_t N, int32_t d, int32_t V, int32_t dtype,
                     float* out_logp, float* out_lse, float* out_entropy, void* workspace,
                     size_t workspace_bytes, void* stream) {
  if (!hidden || !lm_head_w || !target_ids || !out_logp) return MRL_ERR_NULL;
  int rc = check_common(N, d, V, dtype);
  if (rc != MRL_OK) return rc;
  if (N == 0) return MRL_OK;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return MRL_ERR_WORKSPACE;
  const bool entropy = out_entropy != nullptr;
  Layout L;
  rc = pick_chunk(N, 0, d, V, dtype, 0, false, workspace_bytes, L, entropy);
  if (rc != MRL_OK) return rc;
  rc = check_device();
  if (rc != MRL_OK) return rc;

  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool bf16 = dtype == MRL_BF16;
  void* ws = workspace;
  int32_t* row_index = at<int32_t>(ws, L.row_index);
  int64_t* n_scored = at<int64_t>(ws, L.counters);
  {
    Scope sc(MRL_PROF_PREP, s);
    PrepOut po = {row_index, n_scored, n_scored + 1, at<int32_t>(ws, L.block_counts)};
    launch_prep(token_mask, target_ids, N, V, po, s);
    launch_zero_unscored(token_mask, target_ids, N, V, d, out_logp, out_lse, nullptr, 0, s);
    if (entropy) launch_zero_unscored(token_mask, target_ids, N, V, d, out_entropy, nullptr, nullptr, 0, s);
    launch_target_logit(hidden, lm_head_w, target_ids, row_index, n_scored, N, d, bf16, at<float>(ws, L.zt), s);
    if (L.Wp != 0) launch_gather_rows_b16(lm_head_w, d, nullptr, at<void>(ws, L.Wp), L.ldh, V, nullptr, 0, 0, d, L.dp, s);
  }
  for (int64_t c = 0; c < L.n_chunks; ++c) {
    const int64_t c0 = c * L.chunk_rows;
    forward_chunk(hidden, lm_head_w, d, V, bf16, L, ws, c0, false, s, entropy);
    Scope sc(MRL_PROF_ROW_EPI, s);
    RowEpiArgs e = {};
    e.part_max = bf16 ? nullptr : at<float>(ws, L.part_max); e.part_sum = at<float>(ws, L.part_sum);
    e.part_ez = entropy ? at<float>(ws, L.part_ez) : nullptr; e.out_entropy = out_entropy;
    e.n_partials = L.n_partials; e.chunk_rows = L.chunk_rows;
    e.zt = at<float>(ws, L.zt); e.row_index = row_index; e.n_scored = n_scored; e.chunk_start = c0;
    e.out_logp = out_logp; e.out_lse = out_lse;
    launch_row_epilogue(e, s);
  }
  return last_error();
}

int mrl_token_logprobs(const void* hidden, const void* lm_head_w, const int32_t* target_ids,
                       const uint8_t* token_mask, int64_t N, int32_t d, int32_t V, int32_t dtype,
                       float* out_logp, float* out_lse, void* workspace, size_t workspace_bytes,
                       void* stream) {
  return mrl_token_scores(hidden, lm_head_w, target_ids, token_mask, N, d, V, dtype, out_logp, out_lse,
                          nullptr, workspace, workspace_bytes, stream);
}

int mrl_token_logprobs_static(const void* hidden, const void* lm_head_w, const int32_t* target_ids,
                              const uint8_t* token_mask, int64_t N, int32_t d, int32_t V, int32_t dtype,
                              float* out_logp, float* out_lse, void* stream) {
  if (!hidden || !lm_head_w || !target_ids || !out_logp) return MRL_ERR_NULL;
  int rc = check_common(N, d, V, dtype);
  if (rc != MRL_OK) return rc;
  if (N == 0) return MRL_OK;
  // the size check needs no device: the same rule picks the pass size inside the call below
  Layout L;
  if (pick_chunk(N, 0, d, V, dtype, 0, false, MRL_STATIC_SCRATCH_BYTES, L) != MRL_OK) return MRL_ERR_SCRATCH_LIMIT;
  rc = check_device();
  if (rc != MRL_OK) return rc;
  void* ptr = static_scratch_ptr();
  if (ptr == nullptr) return MRL_ERR_DEVICE;
  return mrl_token_scores(hidden, lm_head_w, target_ids, token_mask, N, d, V, dtype, out_logp, out_lse,
                          nullptr, ptr, MRL_STATIC_SCRATCH_BYTES, stream);
}

// --------------------------------------------------------------------------- (2)
int mrl_group_advantages(const float* rewards, const int32_t* group_id, const uint8_t* in_stats,
                         const uint8_t* scored, const uint8_t* is_own, const float* baseline_shift,
                         int64_t B, int32_t G, int32_t adv_mode, float eps_norm, int32_t ddof, float mix_alpha,
                         float neg_thresh, float pos_thresh, float* out_adv, float* out_group_mean,
                         float* out_group_std, uint8_t* out_flags, void* stream) {
  if (!rewards || !group_id || !out_adv) return MRL_ERR_NULL;
  if (B < 0 || B > kMaxSlots || G <= 0 || G > (1 << 24)) return MRL_ERR_SHAPE;
  if (adv_mode < MRL_ADV_CENTER || adv_mode > MRL_ADV_BATCH_ZN) return MRL_ERR_CONFIG;
  if (!(eps_norm >= 0.f) || (ddof != 0 && ddof != 1) || !(mix_alpha >= 0.f && mix_alpha <= 1.f))
    return MRL_ERR_CONFIG;
  if (B == 0) return MRL_OK;
  const int rc = check_device();
  if (rc != MRL_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  Scope sc(MRL_PROF_ADV, s);
  launch_group_advantages(rewards, group_id, in_stats, scored, is_own, baseline_shift, B, G, adv_mode, eps_norm, ddof,
                          mix_alpha, neg_thresh, pos_thresh, out_adv, out_group_mean, out_group_std,
                          out_flags, s);
  return last_error();
}

// --------------------------------------------------------------------------- (3)
size_t mrl_grpo_loss_workspace(int64_t B, int32_t T, int32_t d, int32_t V, int32_t dtype,
                               const mrl_loss_config* cfg) {
  if (B < 0 || T <= 0) return 0;
  const int64_t N = B * (int64_t)T;
  if (check_common(N, d, V, dtype) != MRL_OK) return 0;
  int chunk = default_chunk(N, dtype);
  if (cfg != nullptr) {
    if (check_cfg(cfg) != MRL_OK) return 0;
    if (cfg->chunk_rows > 0) chunk = cfg->chunk_rows;
  }
  return make_layout(N, B, d, V, dtype, chunk, true).total;
}

int mrl_grpo_loss_fwd_bwd(const void* hidden, const void* lm_head_w, const int32_t* target_ids,
                          const uint8_t* token_mask, const float* behav_logp, const float* ref_logp,
                          const float* seq_adv, const int32_t* group_id, const uint8_t* seq_kind,
                          int64_t B, int32_t T, int32_t G, int32_t d, int32_t V, int32_t dtype,
                          const mrl_loss_config* cfg, float* out_logp, void* out_dH, float* out_dW,
                          mrl_loss_stats* out_stats, void* workspace, size_t workspace_bytes,
                          void* stream) {
  if (!hidden || !lm_head_w || !target_ids || !token_mask || !behav_logp || !seq_adv || !group_id ||
      !cfg || !out_logp || !out_stats)
    return MRL_ERR_NULL;
  if (B <= 0 || T <= 0) return MRL_ERR_SHAPE;
  const int64_t N = B * (int64_t)T;
  int rc = check_common(N, d, V, dtype);
  if (rc != MRL_OK) return rc;
  if (G <= 0 || (B > 0 && G > B)) return MRL_ERR_SHAPE;
  rc = check_cfg(cfg);
  if (rc != MRL_OK) return rc;
  if (cfg->kl_beta > 0.f && !ref_logp) return MRL_ERR_NULL;
  if (dtype == MRL_F32 && out_dH && cfg->dh_dtype != MRL_F32) return MRL_ERR_CONFIG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return MRL_ERR_WORKSPACE;
  Layout L;
  rc = pick_chunk(N, B, d, V, dtype, cfg->chunk_rows, true, workspace_bytes, L);
  if (rc != MRL_OK) return rc;
  rc = check_device();
  if (rc != MRL_OK) return rc;

  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool bf16 = dtype == MRL_BF16;
  const bool bwd = out_dH != nullptr || out_dW != nullptr;
  const int es = bf16 ? 2 : 4;
  void* ws = workspace;
  int32_t* row_index = at<int32_t>(ws, L.row_index);
  int64_t* n_scored = at<int64_t>(ws, L.counters);
  const float beta = ref_logp ? cfg->kl_beta : 0.f;

  {
    Scope sc(MRL_PROF_PREP, s);
    PrepOut po = {row_index, n_scored, n_scored + 1, at<int32_t>(ws, L.block_counts)};
    launch_prep(token_mask, target_ids, N, V, po, s);
    launch_seq_weights(token_mask, target_ids, group_id, seq_kind, B, T, G, V, cfg->loss_agg,
                       at<int32_t>(ws, L.seq_len), at<float>(ws, L.seq_coef), at<int32_t>(ws, L.group_count),
                       n_scored + 2, s);
    launch_zero_unscored(token_mask, target_ids, N, V, d, out_logp, nullptr, out_dH,
                         cfg->dh_dtype == MRL_BF16 ? 2 : 4, s);
    launch_target_logit(hidden, lm_head_w, target_ids, row_index, n_scored, N, d, bf16, at<float>(ws, L.zt), s);
    if (L.Wp != 0) launch_gather_rows_b16(lm_head_w, d, nullptr, at<void>(ws, L.Wp), L.ldh, V, nullptr, 0, 0, d, L.dp, s);
  }
  if (cfg->debug_sync) {
    // debugging aid: wait for the preparation kernels and turn the device-side range counters
    // into error codes before any further work is enqueued
    int64_t counters[3] = {0, 0, 0};
    if (hipStreamSynchronize(s) != hipSuccess ||
        hipMemcpy(counters, n_scored, sizeof(counters), hipMemcpyDeviceToHost) != hipSuccess) {
      (void)hipGetLastError();
      return MRL_ERR_DEVICE;
    }
    if (counters[1] != 0) return MRL_ERR_TARGET_RANGE;
    if (counters[2] != 0) return MRL_ERR_GROUP_RANGE;
  }
  if (out_dH) {
    Scope sc(MRL_PROF_CONVERT, s);
    if (bf16)
      launch_transpose(L.Wp != 0 ? at<void>(ws, L.Wp) : lm_head_w, L.Wp != 0 ? L.ldh : d, nullptr, nullptr,
                       at<void>(ws, L.Wt), L.ldz, V, nullptr, 0, 0, L.dp, L.Vp, es, s);
    else
      launch_transpose(lm_head_w, d, nullptr, nullptr, at<void>(ws, L.Wt), L.ldz, V, nullptr, 0, 0, d, L.Vp, es, s);
  }
  int64_t n_passes = L.n_chunks;
  if (cfg->scored_rows_hint > 0) {
    const int64_t by_hint = (cfg->scored_rows_hint + L.chunk_rows - 1) / L.chunk_rows;
    n_passes = by_hint < n_passes ? by_hint : n_passes;
  }
  if (cfg->ratio_level != 0) {
    // Response-level ratio: a response may span several passes, so the log-probs of all rows are
    // computed first (forward only, no stash), then summed per response; the main loop below
    // recomputes them (same bits) on its way to the gradients.
    for (int64_t c = 0; c < n_passes; ++c) {
      const int64_t c0 = c * L.chunk_rows;
      forward_chunk(hidden, lm_head_w, d, V, bf16, L, ws, c0, false, s);
      Scope sc(MRL_PROF_ROW_EPI, s);
      RowEpiArgs e = {};
      e.part_max = bf16 ? nullptr : at<float>(ws, L.part_max); e.part_sum = at<float>(ws, L.part_sum);
      e.n_partials = L.n_partials; e.chunk_rows = L.chunk_rows;
      e.zt = at<float>(ws, L.zt); e.row_index = row_index; e.n_scored = n_scored; e.chunk_start = c0;
      e.out_logp = out_logp;
      launch_row_epilogue(e, s);
    }
    Scope sc(MRL_PROF_ROW_EPI, s);
    launch_seq_log_ratio(token_mask, target_ids, out_logp, behav_logp, B, T, V, cfg->ratio_level,
                         at<float>(ws, L.seq_expo), s);
  }
  for (int64_t c = 0; c < n_passes; ++c) {
    const int64_t c0 = c * L.chunk_rows;
    forward_chunk(hidden, lm_head_w, d, V, bf16, L, ws, c0, bwd, s);
    {
      Scope sc(MRL_PROF_ROW_EPI, s);
      RowEpiArgs e = {};
      e.part_max = bf16 ? nullptr : at<float>(ws, L.part_max); e.part_sum = at<float>(ws, L.part_sum);
      e.n_partials = L.n_partials; e.chunk_rows = L.chunk_rows;
      e.zt = at<float>(ws, L.zt); e.row_index = row_index; e.n_scored = n_scored; e.chunk_start = c0;
      e.behav_logp = behav_logp; e.ref_logp = beta > 0.f ? ref_logp : nullptr; e.seq_adv = seq_adv;
      e.seq_coef = at<float>(ws, L.seq_coef); e.seq_kind = seq_kind; e.T = T;
      e.seq_expo = cfg->ratio_level != 0 ? at<float>(ws, L.seq_expo) : nullptr;
      e.seq_len = at<int32_t>(ws, L.seq_len); e.ratio_level = cfg->ratio_level;
      e.eps_lo = cfg->clip_eps_low; e.eps_hi = cfg->clip_eps_high; e.beta = beta; e.lambda = cfg->sgt_lambda;
      e.out_logp = out_logp; e.out_lse = nullptr;
      e.lse_c = at<float>(ws, L.lse_c); e.g_c = at<float>(ws, L.g_c);
      if (bf16 && bwd) {
        e.row_scale = at<float>(ws, L.row_scale); e.estash = at<uint16_t>(ws, L.Z); e.lde = L.ldz;
        e.targets = target_ids;
      }
      e.loss_partials = at<double>(ws, L.loss_partials);
      e.partial_block_offset = c * row_epilogue_blocks(L.chunk_rows);
      launch_row_epilogue(e, s);
    }
    if (!bwd) continue;
    {
      Scope sc(MRL_PROF_CONVERT, s);
      if (bf16) {
        // the stash already holds the backward operand; only the ragged end of the last pass needs clearing
        launch_zero_stash_tail(at<void>(ws, L.Z), L.ldz, n_scored, c0, L.chunk_rows, (int)L.Vp, s);
      } else {
        launch_convert_f32(at<float>(ws, L.Z), L.ldz, at<float>(ws, L.Pt), L.ldr, at<float>(ws, L.lse_c),
                           at<float>(ws, L.g_c), target_ids, row_index, n_scored, c0, L.chunk_rows, V, s);
      }
      if (out_dW && bf16)   // from the pass's gathered rows, each times its row scale
        launch_transpose(at<void>(ws, L.Hc), L.ldh, nullptr, at<float>(ws, L.row_scale) + c0, at<void>(ws, L.Ht), L.ldr,
                         0, n_scored, c0, L.chunk_rows, L.dp, L.chunk_rows, es, s);
      else if (out_dW)
        launch_transpose(hidden, d, row_index + c0, nullptr, at<void>(ws, L.Ht), L.ldr, 0, n_scored, c0,
                         L.chunk_rows, d, L.chunk_rows, es, s);
    }
    if (out_dH) {
      Scope sc(MRL_PROF_GEMM_DH, s);
      if (bf16) {
        launch_gemm_dh_bf16(at<void>(ws, L.Z), L.ldz, at<void>(ws, L.Wt), L.ldz, row_index,
                            at<float>(ws, L.row_scale), n_scored, c0, L.chunk_rows, (int)L.Vp, d, out_dH,
                            cfg->dh_dtype == MRL_F32, s);
      } else {
        GemmF32Args g = {};
        g.A = at<float>(ws, L.Z); g.lda = L.ldz; g.a_rows = nullptr;
        g.B = at<float>(ws, L.Wt); g.ldb = L.ldz;
        g.C = static_cast<float*>(out_dH); g.ldc = d; g.c_rows = row_index + c0;
        g.M = L.chunk_rows; g.N = d; g.K = V;
        g.n_scored = n_scored; g.chunk_start = c0; g.chunk_rows = L.chunk_rows;
        g.m_dynamic = 1; g.k_dynamic = 0; g.accumulate = 0;
        launch_gemm_f32(g, s);
      }
    }
    if (out_dW) {
      Scope sc(MRL_PROF_GEMM_DW, s);
      const int overwrite = (c == 0 && !cfg->accumulate_dw) ? 1 : 0;
      if (bf16) {
        launch_gemm_dw_bf16(at<void>(ws, L.Z), L.ldz, at<void>(ws, L.Ht), L.ldr, n_scored, c0,
                            L.chunk_rows, V, d, out_dW, overwrite, at<float>(ws, L.dw_tail), s);
      } else {
        GemmF32Args g = {};
        g.A = at<float>(ws, L.Pt); g.lda = L.ldr; g.a_rows = nullptr;
        g.B = at<float>(ws, L.Ht); g.ldb = L.ldr;
        g.C = out_dW; g.ldc = d; g.c_rows = nullptr;
        g.M = V; g.N = d; g.K = L.chunk_rows;
        g.n_scored = n_scored; g.chunk_start = c0; g.chunk_rows = L.chunk_rows;
        g.m_dynamic = 0; g.k_dynamic = 1; g.accumulate = !overwrite;
        launch_gemm_f32(g, s);
      }
    }
  }
  {
    Scope sc(MRL_PROF_FINAL, s);
    launch_finalize(at<double>(ws, L.loss_partials), n_passes * row_epilogue_blocks(L.chunk_rows), n_scored,
                    n_scored + 1, beta, cfg->sgt_lambda, n_passes * (int64_t)L.chunk_rows, row_index, out_logp,
                    out_stats, s);
  }
  return last_error();
}

}  // extern "C"
