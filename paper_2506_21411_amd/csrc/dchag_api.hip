// C ABI of the D-CHAG forward library: argument validation, workspace layout, the host-side
// level scheduler, and kernel launches.  Every step of the path runs in the HIP kernels of
// this directory; there is no CPU fallback.
#include "../../include/dchag.h"

#include <hip/hip_runtime.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>
#include <unordered_map>
#include <vector>

#include "dchag_dev.h"
#include "k_generic.h"
#include "k_mfma.h"
#include "k_fused.h"
#include "k_train.h"
#include "k_yardstick.h"

using namespace dchag;

// Workspace of dchag_aggregate_level_static: lives in the code object, so that call allocates nothing.  In host code
// this name is only a handle for hipGetSymbolAddress; the kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[DCHAG_STATIC_SCRATCH_BYTES];

namespace {

// Debugging switches (environment variables DCHAG_*): read ONCE, when the library is loaded, into this table; the
// calls only look the table up, so the environment of a running process cannot change how a call and the
// dchag_workspace_bytes that sized its workspace split the work.  dchag_debug_reload() reads them again (tests).
enum Switch {
  SW_COLSUM,
  SW_COMPOSE_VALU,
  SW_DZ_PT,
  SW_DZ_VALU,
  SW_FIRST_LEVEL_REGS,
  SW_FIRST_LEVEL_SPLIT,
  SW_FOLD_VALUE_GEMM,
  SW_GEMM,
  SW_GEMM_GENERIC,
  SW_GEMM_SCALAR_STORES,
  SW_GENERIC_LEVEL,
  SW_GENERIC_TOKENIZE,
  SW_LINEAR_SMALL_REGS,
  SW_LINEAR_TOKENS,
  SW_MFMA_TILE,
  SW_MIX_NARROW,
  SW_PIXEL_SCORES_TWO_KERNELS,
  SW_RING_SHAPE,
  SW_RPART_VALU,
  SW_SCORES_ONE_KERNEL,
  SW_SCORES_PER_QUAD,
  SW_TOKENIZE_PER_TILE,
  SW_TOKENS_UNFUSED,
  SW_TOKEN_SCORES,
  SW_VAGG_SPLIT,
  SW_VALUE_UNFOLDED,
  SW_COUNT
};
struct SwitchTable {
  bool set[SW_COUNT];
  char value[SW_COUNT][16];
  void read() {
    static const char* const names[SW_COUNT] = {
    "DCHAG_COLSUM",
    "DCHAG_COMPOSE_VALU",
    "DCHAG_DZ_PT",
    "DCHAG_DZ_VALU",
    "DCHAG_FIRST_LEVEL_REGS",
    "DCHAG_FIRST_LEVEL_SPLIT",
    "DCHAG_FOLD_VALUE_GEMM",
    "DCHAG_GEMM",
    "DCHAG_GEMM_GENERIC",
    "DCHAG_GEMM_SCALAR_STORES",
    "DCHAG_GENERIC_LEVEL",
    "DCHAG_GENERIC_TOKENIZE",
    "DCHAG_LINEAR_SMALL_REGS",
    "DCHAG_LINEAR_TOKENS",
    "DCHAG_MFMA_TILE",
    "DCHAG_MIX_NARROW",
    "DCHAG_PIXEL_SCORES_TWO_KERNELS",
    "DCHAG_RING_SHAPE",
    "DCHAG_RPART_VALU",
    "DCHAG_SCORES_ONE_KERNEL",
    "DCHAG_SCORES_PER_QUAD",
    "DCHAG_TOKENIZE_PER_TILE",
    "DCHAG_TOKENS_UNFUSED",
    "DCHAG_TOKEN_SCORES",
    "DCHAG_VAGG_SPLIT",
    "DCHAG_VALUE_UNFOLDED"};
    for (int i = 0; i < SW_COUNT; ++i) {
      const char* e = getenv(names[i]);
      set[i] = e != nullptr;
      value[i][0] = 0;
      if (e) {
        strncpy(value[i], e, sizeof(value[i]) - 1);
        value[i][sizeof(value[i]) - 1] = 0;
      }
    }
  }
  SwitchTable() { read(); }
};
SwitchTable g_switches;
// The value of a switch, or nullptr when it is not set.
inline const char* dbg(Switch s) { return g_switches.set[s] ? g_switches.value[s] : nullptr; }

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline size_t elem_size(dchag_dtype dt) { return dt == DCHAG_F32 ? 4 : 2; }
inline bool misaligned(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u); }
inline int groups_of(int c_in, int g) { return (c_in + g - 1) / g; }

// The bf16 MFMA path of a level needs 256-wide column slices that hold whole heads or lie inside one.
bool fast_level(dchag_dtype dt, int D, int heads) {
  if (dt != DCHAG_BF16 || D % 256 || heads > 64) return false;
  const int dh = D / heads;
  return dh % 32 == 0 && (256 % dh == 0 || dh % 256 == 0);
}

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// Workspace of one aggregation level, carved in this order (every piece 256-byte aligned).
// Fast path: alpha holds scores, then softmax weights, as [B][G][gpad][heads][Np] floats.
// Generic path: s holds scores [B,Cin,N,heads], v the projected values [B,Cin,N,D].
struct LevelWs {
  size_t qp, mf, mb, alpha, s, v, o, vpart, total;
};

int compute_units();

// Items the value GEMM of a level deals a group's chunks of 8 channels to, so that a level of few groups (the flat
// baseline, the top of a hierarchy) still fills the chip: doubled while there are fewer than two items per compute
// unit, never more than the chunks of the smallest group, at most 8.  DCHAG_VAGG_SPLIT overrides (still clamped).
int vagg_splits(int B, int Cin, int N, int D, int g) {
  const int G = groups_of(Cin, g);
  const int last = Cin - (G - 1) * g;
  const int nch_min = (std::min(g, last) + 7) / 8;
  const long items = (long)(D / 256) * ((N + 31) / 32) * B * G;
  int S = 1;
  if (const char* e = dbg(SW_VAGG_SPLIT)) S = std::max(1, atoi(e));
  else while (items * S < 2L * compute_units() && S < 8) S *= 2;
  while (S > nch_min) S >>= 1;
  return std::max(S, 1);
}

LevelWs level_ws(dchag_dtype dt, int B, int Cin, int N, int D, int heads, int g) {
  const int G = groups_of(Cin, g);
  const size_t es = elem_size(dt);
  const bool fast = fast_level(dt, D, heads) && !dbg(SW_GENERIC_LEVEL);
  LevelWs w{};
  size_t off = 0;
  w.qp = off; off += align_up((size_t)G * D * 4);
  w.mf = off; off += align_up((size_t)G * heads * D * 4);
  w.mb = off; off += align_up((size_t)G * heads * D * 2);
  if (fast) {
    w.alpha = off; off += align_up((size_t)B * G * round_up(g, 8) * heads * round_up(N, 32) * 4);
  } else {
    w.s = off;  off += align_up((size_t)B * Cin * N * heads * 4);
    w.v = off;  off += align_up((size_t)B * Cin * N * D * es);
  }
  w.o = off;  off += align_up((size_t)B * G * N * D * es);
  if (fast) {
    const int S = vagg_splits(B, Cin, N, D, g);
    w.vpart = off;
    if (S > 1) off += align_up((size_t)S * B * G * N * D * 4);
  }
  w.total = off;
  return w;
}

struct ForwardWs {
  size_t tokens, ping, pong, level, ms, msb, cs, mft, prep[16], total;
};

// Projected query, folded keys (fp32 and bf16) of one level, prepared for all levels by one launch at the start of a
// forward call: qp, mf, mb in this order inside the level's prep block.
inline size_t prep_bytes(int G, int D, int heads) {
  return align_up((size_t)G * D * 4) + align_up((size_t)G * heads * D * 4) + align_up((size_t)G * heads * D * 2);
}
struct PrepBufs {
  float *Qp, *Mf;
  bf16* Mb;
};
inline PrepBufs prep_bufs(unsigned char* base, int G, int D, int heads) {
  PrepBufs p;
  p.Qp = reinterpret_cast<float*>(base);
  p.Mf = reinterpret_cast<float*>(base + align_up((size_t)G * D * 4));
  p.Mb = reinterpret_cast<bf16*>(base + align_up((size_t)G * D * 4) + align_up((size_t)G * heads * D * 4));
  return p;
}

// group_sizes has n_levels entries; returns total = 0 when the chain does not end in one group.
ForwardWs forward_ws(dchag_dtype dt, int B, int C, int N, int pp, int D, int heads, int n_levels,
                     const int32_t* group_sizes) {
  ForwardWs w{};
  const size_t es = elem_size(dt);
  size_t off = 0;
  w.tokens = off; off += align_up((size_t)B * C * N * D * es);
  int c_in = C;
  size_t lvl_max = 0, inter_max = 0;
  for (int l = 0; l < n_levels; ++l) {
    const int g = group_sizes[l];
    if (g < 1) return ForwardWs{};
    const size_t t = level_ws(dt, B, c_in, N, D, heads, g).total;
    if (t > lvl_max) lvl_max = t;
    c_in = groups_of(c_in, g);
    if (l + 1 < n_levels) {
      const size_t it = align_up((size_t)B * c_in * N * D * es);
      if (it > inter_max) inter_max = it;
    }
  }
  if (c_in != 1) return ForwardWs{};
  w.ping = off; off += inter_max;
  w.pong = off; off += inter_max;
  w.level = off; off += lvl_max;
  w.ms = off; off += align_up((size_t)C * heads * pp * 4);   // composed level-1 score weights, fp32 and bf16
  w.msb = off; off += align_up((size_t)C * heads * pp * 2);
  w.cs = off; off += align_up((size_t)C * heads * 4);
  w.mft = off; off += align_up((size_t)groups_of(C, group_sizes[0]) * D * heads * 4);
  c_in = C;
  for (int l = 0; l < n_levels; ++l) {
    const int G = groups_of(c_in, group_sizes[l]);
    w.prep[l] = off; off += prep_bytes(G, D, heads);
    c_in = G;
  }
  w.total = off;
  return w;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? DCHAG_OK : DCHAG_ERR_LAUNCH; }

// Optional stage timing (dchag_profile_begin / dchag_profile_end): an event pair per launch.
struct StageRecord {
  hipEvent_t start, stop;
  int stage, level;
};
bool g_profiling = false;
int g_level = 0;
std::vector<StageRecord> g_records;
// The level a stage record is filed under; written only while a profile is being taken.
inline void set_level(int level) {
  if (g_profiling) g_level = level;
}

struct StageTimer {
  hipStream_t st;
  bool on;
  StageRecord rec;
  StageTimer(int stage, hipStream_t s) : st(s), on(g_profiling) {
    if (!on) return;
    rec.stage = stage;
    rec.level = g_level;
    if (hipEventCreate(&rec.start) != hipSuccess || hipEventCreate(&rec.stop) != hipSuccess) {
      on = false;
      return;
    }
    (void)hipEventRecord(rec.start, st);
  }
  ~StageTimer() {
    if (!on) return;
    (void)hipEventRecord(rec.stop, st);
    g_records.push_back(rec);
  }
};

// Compute units of the CURRENT device (looked up once per device; 256 without a device).
constexpr int kMaxDevices = 64;
int compute_units() {
  static std::atomic<int> cus[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  int n = cus[dev].load(std::memory_order_relaxed);
  if (n) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < kXcds) n = 256;
  cus[dev].store(n, std::memory_order_relaxed);
  return n;
}

// Raises a kernel's dynamic-LDS limit to at least `bytes`, once per (device, kernel): later launches only look the
// table up.  Returns 0 or DCHAG_ERR_LAUNCH.
int ensure_dynamic_lds(const void* kernel, int bytes) {
  static std::mutex mu;
  static std::unordered_map<const void*, int> done[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DCHAG_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(mu);
  auto it = done[dev].find(kernel);
  if (it != done[dev].end() && it->second >= bytes) return DCHAG_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return DCHAG_ERR_LAUNCH;
  done[dev][kernel] = bytes;
  return DCHAG_OK;
}

bool force_generic() {
  // DCHAG_GEMM=generic routes the bf16 projections through the fp32-FMA tile kernel (debug aid).
  const char* e = dbg(SW_GEMM);
  return e && strcmp(e, "generic") == 0;
}

// ------------------------------------------------------------------------------------------
// launches
// ------------------------------------------------------------------------------------------
template <typename T>
int launch_tokenize(int B, int C, int H, int W, int p, int D, const T* x, const T* We, const T* be,
                    const T* ce, T* tokens, hipStream_t st) {
  constexpr int TP = 16;
  const int N = (H / p) * (W / p);
  dim3 grid((N + TP - 1) / TP, C, B);
  const size_t lds = (size_t)TP * p * p * sizeof(float);
  StageTimer tm(DCHAG_STAGE_TOKENIZE, st);
  k_tokenize_generic<T, TP><<<grid, 256, lds, st>>>(C, H, W, p, D, x, We, be, ce, tokens);
  return launch_status();
}

int launch_tokenize_mfma(int B, int C, int H, int W, int p, int D, const bf16* x, const bf16* We, const bf16* be,
                         const bf16* ce, bf16* tokens, hipStream_t st) {
  const int N = (H / p) * (W / p);
  const int ks = p * p / 16;
  if ((ks == 1 || ks == 2 || ks == 4) && p * p == 16 * ks && D % 256 == 0 && !dbg(SW_TOKENIZE_PER_TILE)) {
    // weight-stationary form: enough blocks for about eight per compute unit, each walking `per` tiles
    const int T = B * ((N + 127) / 128);
    const long base = (long)(D / 256) * C;
    int ts = (int)((8L * compute_units() + base - 1) / base);
    ts = ts < 1 ? 1 : (ts > T ? T : ts);
    const int per = (T + ts - 1) / ts;
    ts = (T + per - 1) / per;
    const size_t wlds = (size_t)2 * 128 * (p * p * 2 + 16);
    auto wk = ks == 1 ? k_tokenize_ws<1> : ks == 2 ? k_tokenize_ws<2> : k_tokenize_ws<4>;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(wk), (int)wlds)) return DCHAG_ERR_LAUNCH;
    StageTimer tm(DCHAG_STAGE_TOKENIZE, st);
    wk<<<dim3(D / 256, C, ts), 256, wlds, st>>>(B, C, H, W, p, D, per, x, We, be, ce, tokens);
    return launch_status();
  }
  const size_t lds = (size_t)128 * (p * p * 2 + 16);
  auto kern = ks == 1 ? k_tokenize_mfma<1> : ks == 2 ? k_tokenize_mfma<2> : ks == 4 ? k_tokenize_mfma<4> : k_tokenize_mfma<0>;
  if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds)) return DCHAG_ERR_LAUNCH;
  StageTimer tm(DCHAG_STAGE_TOKENIZE, st);
  kern<<<dim3((N + 127) / 128, C, B), 256, lds, st>>>(C, H, W, p, D, x, We, be, ce, tokens);
  return launch_status();
}

template <typename T>
int launch_linear_generic(int B, int D, RowBlocks rb, const T* A, const T* Wt, const T* bias, T* Y,
                          hipStream_t st, const T* rowadd = nullptr) {
  dim3 grid((D + 63) / 64, (rb.rows_per_group + 63) / 64, B * rb.G);
  k_linear_generic<T><<<grid, 256, 0, st>>>(D, rb, A, Wt, bias, Y, rowadd);
  return launch_status();
}

template <int BM, int BN, int WM, int WN, int SH>
int launch_linear_mfma_cfg(int B, int D, RowBlocks rb, const bf16* A, const bf16* Wt, const bf16* bias,
                           bf16* Y, hipStream_t st, const bf16* rowadd = nullptr) {
  TileWork tw;
  tw.n_tiles = D / BN;
  tw.m_tiles = (rb.rows_per_group + BM - 1) / BM;
  tw.nb = B;
  tw.total = tw.n_tiles * tw.m_tiles * B * rb.G;
  const int per = (tw.total + kXcds - 1) / kXcds;
  const size_t lds = (size_t)2 * (BM + BN) * 128;
  auto kern = k_linear_mfma<BM, BN, WM, WN, SH>;
  if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds)) return DCHAG_ERR_LAUNCH;
  kern<<<dim3(per * kXcds), dim3(WM * WN * 64), lds, st>>>(D, rb, tw, A, Wt, bias, Y, rowadd);
  return launch_status();
}

int mfma_variant() {
  // DCHAG_MFMA_TILE selects the block tiling of the bf16 projection kernel (tuning aid).
  const char* e = dbg(SW_MFMA_TILE);
  return e ? atoi(e) : 0;
}

template <typename T>
int launch_linear(int B, int D, RowBlocks rb, const T* A, const T* Wt, const T* bias, T* Y, hipStream_t st,
                  const T* rowadd = nullptr);

template <>
int launch_linear<float>(int B, int D, RowBlocks rb, const float* A, const float* Wt, const float* bias,
                         float* Y, hipStream_t st, const float* rowadd) {
  return launch_linear_generic<float>(B, D, rb, A, Wt, bias, Y, st, rowadd);
}

template <>
int launch_linear<bf16>(int B, int D, RowBlocks rb, const bf16* A, const bf16* Wt, const bf16* bias, bf16* Y,
                        hipStream_t st, const bf16* rowadd) {
  if (D % 256 == 0 && !force_generic()) {
    switch (mfma_variant()) {
      case 1: return launch_linear_mfma_cfg<256, 256, 2, 4, 0>(B, D, rb, A, Wt, bias, Y, st, rowadd);
      case 2: return launch_linear_mfma_cfg<256, 128, 2, 2, 0>(B, D, rb, A, Wt, bias, Y, st, rowadd);
      case 3: return launch_linear_mfma_cfg<128, 128, 2, 2, 0>(B, D, rb, A, Wt, bias, Y, st, rowadd);
      case 4: return launch_linear_mfma_cfg<256, 256, 2, 2, 1>(B, D, rb, A, Wt, bias, Y, st, rowadd);
      default: return launch_linear_mfma_cfg<256, 256, 2, 2, 0>(B, D, rb, A, Wt, bias, Y, st, rowadd);
    }
  }
  return launch_linear_generic<bf16>(B, D, rb, A, Wt, bias, Y, st, rowadd);
}

// One aggregation level: weight-only prep, scores, value projection, softmax-weighted sum,
// output projection.
template <typename T>
int run_level(dchag_dtype dt, int B, int Cin, int N, int D, int heads, const dchag_level* lv, const T* zin,
              T* zout, unsigned char* ws, hipStream_t st, const T* rowadd = nullptr) {
  const int g = lv->group_size;
  const int G = groups_of(Cin, g);
  const LevelWs w = level_ws(dt, B, Cin, N, D, heads, g);
  float* Qp = reinterpret_cast<float*>(ws + w.qp);
  float* Mf = reinterpret_cast<float*>(ws + w.mf);
  float* S = reinterpret_cast<float*>(ws + w.s);
  T* V = reinterpret_cast<T*>(ws + w.v);
  T* O = reinterpret_cast<T*>(ws + w.o);
  int rc;

  {
    StageTimer tm(DCHAG_STAGE_QUERY, st);
    k_project_query<T><<<dim3((D + 3) / 4, G), 256, 0, st>>>(
        D, static_cast<const T*>(lv->query), static_cast<const T*>(lv->Wq), static_cast<const T*>(lv->bq), Qp);
    if ((rc = launch_status())) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_FOLD, st);
    k_fold_query_into_key<T><<<dim3((D + 63) / 64, heads, G), 256, 0, st>>>(
        D, heads, static_cast<const T*>(lv->Wk), Qp, Mf, nullptr, nullptr);
    if ((rc = launch_status())) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_SCORES, st);
    const long T_total = (long)B * Cin * N;
    k_scores_generic<T, 8><<<dim3((unsigned)((T_total + 3) / 4)), 256, 0, st>>>(T_total, Cin, N, D, heads, g, zin,
                                                                               Mf, S);
    if ((rc = launch_status())) return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_VPROJ, st);
    RowBlocks rbv{G, Cin * N, g * N};
    if ((rc = launch_linear<T>(B, D, rbv, zin, static_cast<const T*>(lv->Wv), static_cast<const T*>(lv->bv), V, st)))
      return rc;
  }
  {
    StageTimer tm(DCHAG_STAGE_SOFTMAX_AGG, st);
    k_softmax_aggregate_generic<T><<<dim3(N, G, B), 256, 0, st>>>(Cin, N, D, heads, g, S, V, O);
    if ((rc = launch_status())) return rc;
  }
  StageTimer tm(DCHAG_STAGE_OPROJ, st);
  RowBlocks rbo{G, G * N, N};
  return launch_linear<T>(B, D, rbo, O, static_cast<const T*>(lv->Wo), static_cast<const T*>(lv->bo), zout, st,
                          rowadd);
}

int launch_linear_dl(int B, int D, RowBlocks rb, const bf16* A, const bf16* Wt, const bf16* bias, bf16* Y,
                     hipStream_t st, const bf16* rowadd = nullptr) {
  TileWork tw;
  tw.n_tiles = D / kGemmBN;
  tw.m_tiles = (rb.rows_per_group + kGemmBM - 1) / kGemmBM;
  tw.nb = B;
  tw.total = tw.n_tiles * tw.m_tiles * B * rb.G;
  if (tw.total * 2 < compute_units()) {                  // too few 256x256 tiles to fill the chip: 128x128 tiles, and
    if (dbg(SW_LINEAR_SMALL_REGS))                         // loads three slices ahead (the debugging switch keeps the
      return launch_linear_mfma_cfg<128, 128, 2, 2, 1>(B, D, rb, A, Wt, bias, Y, st, rowadd);   // register-staged kernel)
    TileWork ts;
    ts.n_tiles = D / 128;
    ts.m_tiles = (rb.rows_per_group + 127) / 128;
    ts.nb = B;
    ts.total = ts.n_tiles * ts.m_tiles * B * rb.G;
    const int pers = (ts.total + kXcds - 1) / kXcds;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(k_linear_ring), kSmallRingBytes)) return DCHAG_ERR_LAUNCH;
    k_linear_ring<<<dim3(pers * kXcds), dim3(256), kSmallRingBytes, st>>>(D, rb, ts, A, Wt, bias, Y, rowadd);
    return launch_status();
  }
  const int per = (tw.total + kXcds - 1) / kXcds;
  if (ensure_dynamic_lds(reinterpret_cast<const void*>(k_linear_dl), kGemmRingBytes)) return DCHAG_ERR_LAUNCH;
  k_linear_dl<<<dim3(per * kXcds), dim3(512), kGemmRingBytes, st>>>(D, rb, tw, A, Wt, bias, Y, rowadd);
  return launch_status();
}

// Inputs of the first level's score shortcut: scores computed from the pixels through the
// tokenizer weights composed with the folded keys.
struct PixelScores {
  const bf16 *x, *We, *be, *ce;
  int H, W, p;
  float *Ms, *cs, *MfT;
  bf16* Msb;
};

// The first level's scores can come from the pixels when the compose kernel (4 x 4 output tiles, at most 4 per
// lane) and the pixel-score kernel (one 32-wide MFMA column block of heads, 8-pixel operand chunks) tile the shape.
bool pixel_scores_ok(int p, int heads) {
  const int pp = p * p;
  return heads % 4 == 0 && heads <= 32 && pp % 16 == 0 && (p == 4 || p % 8 == 0) && (heads / 4) * (pp / 4) <= 256 &&
         pp <= 256 && !dbg(SW_TOKEN_SCORES);
}

// Projected queries and query-folded keys of n attention levels (bf16, D % 8 == 0) in one launch.
struct KeyPrepJob {
  const dchag_level* lv;
  int G;
  PrepBufs out;
  float* MfT;                      // optional transposed copy of the folded keys
};
int launch_query_keys(int D, int heads, const KeyPrepJob* jobs, int n, hipStream_t st) {
  KeyPrepArgs args{};
  int total = 0;
  args.n_levels = n;
  for (int i = 0; i < n; ++i) {
    const dchag_level* lv = jobs[i].lv;
    args.lv[i] = KeyPrepLevel{static_cast<const bf16*>(lv->query), static_cast<const bf16*>(lv->Wq),
                              static_cast<const bf16*>(lv->bq),    static_cast<const bf16*>(lv->Wk),
                              jobs[i].out.Qp, jobs[i].out.Mf, jobs[i].MfT, jobs[i].out.Mb, total};
    total += jobs[i].G;
  }
  if (total > 65535 || heads > 65535) return DCHAG_ERR_SHAPE;
  StageTimer tm(DCHAG_STAGE_KEY_PREP, st);
  // shares of the columns per (head, group): enough blocks for two per compute unit, whole 512-column passes each
  int shares = 1;
  while ((long)heads * total * shares < 2L * compute_units() && D % (1024 * shares) == 0 && shares < 8) shares *= 2;
  k_query_keys<<<dim3(heads, total, shares), 256, (size_t)(D / heads + 1536) * 4, st>>>(D, heads, args);
  return launch_status();
}

// Weight-only prep, scores and softmax of one level on the bf16 MFMA path: leaves the projected query in
// Qp, the folded keys in Mf / Mb and the softmax weights in alpha, laid out [B][G][gpad][heads][Np].
// alpha_tm (optional): where the softmax weights are also wanted token-major [B,Cin,N,heads]; *tm_done tells whether
// they were written (only the one-kernel pixel route does it; otherwise the caller re-lays alpha).
// phase: 0 = everything; 1 = the weight-only prep alone (Qp, Mf, Mb and, with px, its composed score weights; B, N, zin
// and alpha are not used); 2 = scores and softmax alone, from a prep that is already in those buffers; 3 = everything
// but the projected query and the folded keys, which are already in Qp, Mf, Mb (and px->MfT).
int fast_scores(int B, int Cin, int N, int D, int heads, const dchag_level* lv, const bf16* zin, float* Qp, float* Mf,
                bf16* Mb, float* alpha, hipStream_t st, const PixelScores* px, float* alpha_tm = nullptr,
                bool* tm_done = nullptr, int phase = 0) {
  if (tm_done) *tm_done = false;
  const int g = lv->group_size;
  const int G = groups_of(Cin, g);
  const int gpad = round_up(g, 8), Np = round_up(N, 32);
  int rc;
  if (phase != 2 && phase != 3) {
    const KeyPrepJob job{lv, G, PrepBufs{Qp, Mf, Mb}, px ? px->MfT : nullptr};
    if ((rc = launch_query_keys(D, heads, &job, 1, st))) return rc;
  }
  if (phase == 1 && !px) return DCHAG_OK;
  if (px) {
    StageTimer tm(DCHAG_STAGE_SCORES, st);
    const int pp = px->p * px->p;
    // MFMA form of the weight composition where the shape allows it (DCHAG_COMPOSE_VALU, a debugging aid, keeps
    // the vector-ALU kernel): pp = 16 .. 128 in blocks of 8 pixels, groups that are multiples of the block's channels
    const int cpb = (pp == 16 || pp == 32 || pp == 64 || pp == 128) ? 16 / (pp / 8) : 0;
    const bool compose_mfma = cpb > 0 && g % cpb == 0 && D % 128 == 0 && heads <= 32 && !dbg(SW_COMPOSE_VALU);
    if (compose_mfma && phase != 2) {
      const dim3 cgrid((unsigned)((Cin + cpb - 1) / cpb));
      if (heads <= 16)
        k_compose_score_weights_mfma<1><<<cgrid, 256, 0, st>>>(Cin, D, heads, pp, g, Mf, px->We, px->be, px->ce, px->Ms,
                                                              px->Msb, px->cs);
      else
        k_compose_score_weights_mfma<2><<<cgrid, 256, 0, st>>>(Cin, D, heads, pp, g, Mf, px->We, px->be, px->ce, px->Ms,
                                                              px->Msb, px->cs);
      if ((rc = launch_status())) return rc;
    }
    const int ntiles = (heads / 4) * (pp / 4);
    const int TPL = ntiles <= 64 ? 1 : (ntiles <= 128 ? 2 : 4);
    int DQ = 16384 / pp;                                 // 32 KiB of tokenizer weights per block of d
    while (D % DQ) DQ >>= 1;
    const size_t clds = (size_t)DQ * (pp * 2 + heads * 4 + 4) + (size_t)3 * TPL * 64 * 20 * 4;
    auto compose = TPL == 1 ? k_compose_score_weights<1> : (TPL == 2 ? k_compose_score_weights<2> : k_compose_score_weights<4>);
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(compose), (int)clds)) return DCHAG_ERR_LAUNCH;
    if (!compose_mfma && phase != 2) {
      compose<<<dim3(Cin), 256, clds, st>>>(D, heads, pp, g, DQ, px->MfT, px->We, px->be, px->ce, px->Ms, px->Msb, px->cs);
      if ((rc = launch_status())) return rc;
    }
    if (phase == 1) return DCHAG_OK;
    // scores and softmax in one kernel while a group's scores of 32 patches fit LDS (DCHAG_PIXEL_SCORES_TWO_KERNELS,
    // a debugging aid, keeps them apart)
    const size_t slds = (size_t)std::min(g, Cin) * heads * 33 * 4;
    if (slds <= 150 * 1024 && B <= 65535 && G <= 65535 && !dbg(SW_PIXEL_SCORES_TWO_KERNELS)) {
      auto sk = pp == 64 ? k_scores_pixels_softmax<64> : (pp == 16 ? k_scores_pixels_softmax<16> : k_scores_pixels_softmax<0>);
      if (ensure_dynamic_lds(reinterpret_cast<const void*>(sk), (int)slds)) return DCHAG_ERR_LAUNCH;
      sk<<<dim3((N + 31) / 32, G, B), 256, slds, st>>>(Cin, px->H, px->W, px->p, heads, g, gpad, G, Np, px->x, px->Msb,
                                                      px->cs, alpha_tm ? nullptr : alpha, alpha_tm);
      if ((rc = launch_status())) return rc;
      if (tm_done && alpha_tm) *tm_done = true;
    } else {
      k_scores_pixels<<<dim3((N + 127) / 128, Cin, B), 256, 0, st>>>(Cin, px->H, px->W, px->p, heads, g, gpad, G, Np,
                                                                   px->x, px->Msb, px->cs, alpha);
      if ((rc = launch_status())) return rc;
      k_softmax_alpha<<<dim3((Np + 255) / 256, heads, B * G), 256, 0, st>>>(Cin, N, heads, g, gpad, G, Np, alpha);
      if ((rc = launch_status())) return rc;
    }
  } else {
    StageTimer tm(DCHAG_STAGE_SCORES, st);
    const int NB = (heads + 15) / 16;
    const dim3 grid((N + 15) / 16, G * ((g + 3) / 4), B);
    // group-resident form: folded keys in registers (KI * NB fragments); enough blocks to fill the chip
    const int KI = D / 128, nq = (g + 3) / 4;
    const long base_blocks = (long)((N + 15) / 16) * G * B;
    int qsplit = (int)((8L * compute_units() + base_blocks - 1) / base_blocks);
    qsplit = qsplit < 1 ? 1 : (qsplit > nq ? nq : qsplit);
    const int qper = (nq + qsplit - 1) / qsplit;
    qsplit = (nq + qper - 1) / qper;
    const dim3 ggrid((N + 15) / 16, G * qsplit, B);
#define DCHAG_SCORES_GROUP(NB_, KI_)                                                                         \
  k_scores_group<NB_, KI_><<<ggrid, 256, 0, st>>>(Cin, N, heads, g, gpad, Np, qsplit, qper, zin, Mb, alpha)
    const bool resident = D % 128 == 0 && !dbg(SW_SCORES_PER_QUAD);
    // scores + softmax in one kernel: folded keys of the whole row in registers, raw scores in LDS
    const size_t slds = (size_t)16 * (2 * D + 16) + (size_t)gpad * 2048;
    // DCHAG_SCORES_ONE_KERNEL = 0 / 1 overrides the size heuristic (never the shape limits)
    const char* force = dbg(SW_SCORES_ONE_KERNEL);
    const bool fits = NB <= 1 && D % 256 == 0 && slds <= 150 * 1024;
    const bool one_kernel = fits && (force ? force[0] == '1' : (long)(Np / 32) * G * B >= compute_units());
    if (one_kernel) {
      if (ensure_dynamic_lds(reinterpret_cast<const void*>(k_scores_softmax), (int)slds)) return DCHAG_ERR_LAUNCH;
      k_scores_softmax<<<dim3(Np / 32, G, B), 512, slds, st>>>(Cin, N, D, heads, g, gpad, Np, zin, Mb, alpha);
      if ((rc = launch_status())) return rc;
    } else {
    if (resident && NB <= 1 && KI == 2) DCHAG_SCORES_GROUP(1, 2);
    else if (resident && NB <= 1 && KI == 4) DCHAG_SCORES_GROUP(1, 4);
    else if (resident && NB <= 1 && KI == 8) DCHAG_SCORES_GROUP(1, 8);
    else if (resident && NB <= 1 && KI == 16) DCHAG_SCORES_GROUP(1, 16);
    else if (resident && NB == 2 && KI == 2) DCHAG_SCORES_GROUP(2, 2);
    else if (resident && NB == 2 && KI == 4) DCHAG_SCORES_GROUP(2, 4);
    else if (resident && NB == 2 && KI == 8) DCHAG_SCORES_GROUP(2, 8);
#undef DCHAG_SCORES_GROUP
    else if (NB <= 1)
      k_scores_mfma<1><<<grid, 256, 0, st>>>(Cin, N, D, heads, g, gpad, Np, zin, Mb, alpha);
    else if (NB == 2)
      k_scores_mfma<2><<<grid, 256, 0, st>>>(Cin, N, D, heads, g, gpad, Np, zin, Mb, alpha);
    else
      k_scores_mfma<4><<<grid, 256, 0, st>>>(Cin, N, D, heads, g, gpad, Np, zin, Mb, alpha);
    if ((rc = launch_status())) return rc;
    k_softmax_alpha<<<dim3((Np + 255) / 256, heads, B * G), 256, 0, st>>>(Cin, N, heads, g, gpad, G, Np, alpha);
    if ((rc = launch_status())) return rc;
    }
  }
  return DCHAG_OK;
}

// One aggregation level on the bf16 MFMA path: weight-only prep, scores (MFMA on the tokens, or
// from the pixels at the first level of a forward call), softmax over the group, value projection
// fused with the weighted sum over the group, output projection.
// ready: the level's projected query and folded keys, when a launch at the start of the call has prepared them.
int run_level_fast(int B, int Cin, int N, int D, int heads, const dchag_level* lv, const bf16* zin, bf16* zout,
                   unsigned char* ws, hipStream_t st, const PixelScores* px = nullptr, const bf16* rowadd = nullptr,
                   const PrepBufs* ready = nullptr) {
  const int g = lv->group_size;
  const int G = groups_of(Cin, g);
  const int gpad = round_up(g, 8), Np = round_up(N, 32);
  const LevelWs w = level_ws(DCHAG_BF16, B, Cin, N, D, heads, g);
  float* alpha = reinterpret_cast<float*>(ws + w.alpha);
  bf16* O = reinterpret_cast<bf16*>(ws + w.o);
  int rc;
  const PrepBufs own{reinterpret_cast<float*>(ws + w.qp), reinterpret_cast<float*>(ws + w.mf),
                     reinterpret_cast<bf16*>(ws + w.mb)};
  const PrepBufs& pb = ready ? *ready : own;
  if ((rc = fast_scores(B, Cin, N, D, heads, lv, zin, pb.Qp, pb.Mf, pb.Mb, alpha, st, px, nullptr, nullptr,
                        ready ? 3 : 0)))
    return rc;
  {
    StageTimer tm(DCHAG_STAGE_FUSED_VAGG, st);
    TileWork tw;
    tw.n_tiles = D / kGemmBN;
    tw.m_tiles = (N + 31) / 32;
    tw.nb = B;
    const int S = vagg_splits(B, Cin, N, D, g);
    float* Opart = reinterpret_cast<float*>(ws + w.vpart);
    tw.total = tw.n_tiles * tw.m_tiles * B * G * S;
    const int per = (tw.total + kXcds - 1) / kXcds;
    const int dh = D / heads;
    const int NHS = dh >= kGemmBN ? 1 : kGemmBN / dh;
    const int lds = kGemmRingBytes + 3 * 8 * NHS * 32 * 4;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(k_vagg_mfma), lds)) return DCHAG_ERR_LAUNCH;
    // persistent workgroups: one per compute unit (the LDS ring allows no more), `slots` per XCD
    const int slots = per < compute_units() / kXcds ? per : compute_units() / kXcds;
    k_vagg_mfma<<<dim3(slots * kXcds), dim3(512), lds, st>>>(Cin, N, D, heads, g, gpad, G, Np, tw, slots, zin,
                                                            static_cast<const bf16*>(lv->Wv),
                                                            static_cast<const bf16*>(lv->bv), alpha, O, S, Opart);
    if ((rc = launch_status())) return rc;
    if (S > 1) {
      const long per_split = (long)B * G * N * D, quads = per_split / 4;
      k_vagg_merge<<<dim3((unsigned)((quads + 255) / 256)), 256, 0, st>>>(quads, S, G, N, D, per_split, Opart,
                                                                         static_cast<const bf16*>(lv->bv), O);
      if ((rc = launch_status())) return rc;
    }
  }
  StageTimer tm(DCHAG_STAGE_OPROJ, st);
  RowBlocks rbo{G, G * N, N};
  return launch_linear_dl(B, D, rbo, O, static_cast<const bf16*>(lv->Wo), static_cast<const bf16*>(lv->bo), zout, st,
                          rowadd);
}

// A linear (D-CHAG-L) level: one memory-bound mixing kernel, no workspace.
template <typename T>
int run_level_linear(int B, int Cin, int N, int D, const dchag_level* lv, const T* zin, T* zout, hipStream_t st) {
  const int g = lv->group_size;
  const int G = groups_of(Cin, g);
  constexpr int V = 16 / sizeof(T);
  const long total = (long)N * (D / V);
  StageTimer tm(DCHAG_STAGE_CHANNEL_MIX, st);
  k_channel_mix<T><<<dim3((unsigned)((total + 255) / 256), G, B), 256, 0, st>>>(
      Cin, N, D, g, zin, static_cast<const T*>(lv->Wv), static_cast<const T*>(lv->bv), zout);
  return launch_status();
}

int check_level(const dchag_level* lv) {
  if (!lv) return DCHAG_ERR_NULL;
  if (lv->group_size < 1) return DCHAG_ERR_SHAPE;
  if (lv->kind == DCHAG_LEVEL_LINEAR) {
    if (!lv->Wv) return DCHAG_ERR_NULL;
    if (misaligned(lv->Wv) || misaligned(lv->bv)) return DCHAG_ERR_ALIGN;
    return DCHAG_OK;
  }
  if (lv->kind != DCHAG_LEVEL_ATTENTION) return DCHAG_ERR_SHAPE;
  if (!lv->query || !lv->Wq || !lv->Wk || !lv->Wv || !lv->Wo) return DCHAG_ERR_NULL;
  const void* ps[] = {lv->query, lv->Wq, lv->Wk, lv->Wv, lv->Wo, lv->bq, lv->bk, lv->bv, lv->bo};
  for (const void* p : ps)
    if (misaligned(p)) return DCHAG_ERR_ALIGN;
  return DCHAG_OK;
}

int check_tokenize_shape(int B, int C, int H, int W, int p, int D) {
  if (B < 1 || C < 1 || H < 1 || W < 1 || p < 1 || D < 1) return DCHAG_ERR_SHAPE;
  if (H % p || W % p || D % 8) return DCHAG_ERR_SHAPE;
  if (p > 32 || C > 65535 || B > 65535) return DCHAG_ERR_SHAPE;
  if ((size_t)B * C * (size_t)(H / p) * (W / p) * D >= ((size_t)1 << 40)) return DCHAG_ERR_SHAPE;
  return DCHAG_OK;
}

int check_level_shape(int B, int Cin, int N, int D, int heads, int g) {
  if (B < 1 || Cin < 1 || N < 1 || D < 1 || heads < 1 || g < 1) return DCHAG_ERR_SHAPE;
  if (D % heads || D % 8) return DCHAG_ERR_SHAPE;
  const int G = groups_of(Cin, g);
  if ((long)B * G > 65535 || B > 65535 || G > 65535 || heads > 65535) return DCHAG_ERR_SHAPE;
  if ((long)g * N > (1L << 30) || (long)Cin * N > (1L << 30)) return DCHAG_ERR_SHAPE;
  return DCHAG_OK;
}

// Tokenizer and a linear first level in one kernel (bf16, p*p = 16 or 64, D % 256 == 0): the per-channel tokens never
// reach HBM.  y [B,G,N,D].
inline bool tokenize_mix_ok(dchag_dtype dt, const dchag_level* levels, int pp, int D) {
  return dt == DCHAG_BF16 && levels[0].kind == DCHAG_LEVEL_LINEAR && (pp == 16 || pp == 64) && D % 256 == 0 &&
         !dbg(SW_GENERIC_TOKENIZE);
}
// The ring-buffered kernel of the fused tokenizer + first level takes 8 x 8 patches whose rows, like every weight and
// vector row it streams, are whole 16-byte pieces (DCHAG_FIRST_LEVEL_REGS, a debugging aid, keeps the older kernels).
inline bool aligned16(const void* ptr) { return !(reinterpret_cast<uintptr_t>(ptr) & 15); }
inline bool reduce_ring_ok(int p, int W, int D, const void* x, const void* Wt, const void* v0, const void* v1,
                           const void* v2) {
  return p == 8 && W % 8 == 0 && D % 256 == 0 && aligned16(x) && aligned16(Wt) && aligned16(v0) && aligned16(v1) &&
         aligned16(v2) && !dbg(SW_FIRST_LEVEL_REGS);
}
template <bool ATT, int CFG>
int launch_reduce_ring_cols(int B, int C, int H, int W, int D, int g, int heads, const bf16* x, const bf16* Wt,
                            const bf16* wmix, const bf16* v1, const bf16* v2, const float* alpha, const bf16* bias,
                            bf16* y, hipStream_t st, float* part, size_t part_bytes) {
  typedef RedCfg<CFG> Cfg;
  const int N = (H / 8) * (W / 8), G = groups_of(C, g);
  TileWork tw{};
  tw.n_tiles = D / Cfg::kCols;
  tw.m_tiles = (N + Cfg::kPatches - 1) / Cfg::kPatches;
  tw.nb = B;
  const long total = (long)G * B * tw.m_tiles * tw.n_tiles;
  if (total > (1L << 26)) return DCHAG_ERR_SHAPE;
  tw.total = (int)total;
  const size_t per_split = (size_t)B * G * N * D;
  const int gmin = std::min(g, C - (G - 1) * g);                  // members of the shortest group
  const long fill = 2L * Cfg::kPerCu * compute_units();           // workgroups that give every compute unit two rounds
  int S = 1;
  while (total * S < fill && 2 * S <= std::min(16, gmin)) S *= 2;
  if (const char* e = dbg(SW_FIRST_LEVEL_SPLIT)) S = std::max(1, std::min(std::min(16, gmin), atoi(e)));
  while (S > 1 && (!part || (size_t)S * per_split * 4 > part_bytes)) S >>= 1;
  const int per = (int)((total * S + kXcds - 1) / kXcds);
  if (ensure_dynamic_lds(reinterpret_cast<const void*>(k_tokenize_reduce_ring<ATT, CFG>), Cfg::kLdsBytes)) return DCHAG_ERR_LAUNCH;
  k_tokenize_reduce_ring<ATT, CFG><<<dim3((unsigned)(per * kXcds)), Cfg::kThreads, Cfg::kLdsBytes, st>>>(
      C, H, W, D, g, G, heads, round_up(g, 8), round_up(N, 32), tw, x, Wt, wmix, v1, v2, alpha, bias, y, S, part);
  int rc = launch_status();
  if (rc || S == 1) return rc;
  const long quads = (long)per_split / 4;
  k_vagg_merge<<<dim3((unsigned)((quads + 255) / 256)), 256, 0, st>>>(quads, S, G, N, D, (long)per_split, part, bias, y);
  return launch_status();
}

// part / part_bytes: optional fp32 scratch for partial sums; with it, and too few tiles to give every compute unit two
// rounds of workgroups, a group's members are dealt to up to 16 workgroups per tile (DCHAG_FIRST_LEVEL_SPLIT overrides
// the count).  Workgroups of 128 patches x 256 columns, one per compute unit, three stages (DCHAG_RING_SHAPE = 1:
// 128 x 128, two per compute unit, two stages).
template <bool ATT>
int launch_reduce_ring(int B, int C, int H, int W, int D, int g, int heads, const bf16* x, const bf16* Wt,
                       const bf16* wmix, const bf16* v1, const bf16* v2, const float* alpha, const bf16* bias, bf16* y,
                       hipStream_t st, float* part = nullptr, size_t part_bytes = 0) {
  const char* e = dbg(SW_RING_SHAPE);
  if (e && atoi(e) == 1)
    return launch_reduce_ring_cols<ATT, 1>(B, C, H, W, D, g, heads, x, Wt, wmix, v1, v2, alpha, bias, y, st, part,
                                           part_bytes);
  return launch_reduce_ring_cols<ATT, 0>(B, C, H, W, D, g, heads, x, Wt, wmix, v1, v2, alpha, bias, y, st, part,
                                         part_bytes);
}

int tokenize_mix_forward(int B, int C, int H, int W, int p, int D, const void* x, const void* We, const void* be,
                         const void* ce, const dchag_level* lv, bf16* y, hipStream_t st) {
  const int N = (H / p) * (W / p), pp = p * p, g = lv->group_size, G = groups_of(C, g);
  if (reduce_ring_ok(p, W, D, x, We, lv->Wv, be, ce)) {
    StageTimer tm(DCHAG_STAGE_TOKENIZE_MIX, st);
    return launch_reduce_ring<false>(B, C, H, W, D, g, 1, static_cast<const bf16*>(x), static_cast<const bf16*>(We),
                                     static_cast<const bf16*>(lv->Wv), static_cast<const bf16*>(be),
                                     static_cast<const bf16*>(ce), nullptr, static_cast<const bf16*>(lv->bv), y, st);
  }
  // 128 patches per workgroup (eight wavefronts) while that leaves a workgroup per compute unit, else 64 (four);
  // DCHAG_MIX_NARROW (debugging aid) keeps the 64-patch kernel
  const bool wide = N >= 128 && (long)((N + 127) / 128) * (D / 256) * G * B >= compute_units() && !dbg(SW_MIX_NARROW);
  const int PB = wide ? 128 : 64;
  const size_t lds = (size_t)2 * PB * (pp * 2 + 16);
  auto mixk = wide ? (pp == 16 ? k_tokenize_mix_wide<1> : k_tokenize_mix_wide<4>)
                   : (pp == 16 ? k_tokenize_mix_mfma<1> : k_tokenize_mix_mfma<4>);
  if (ensure_dynamic_lds(reinterpret_cast<const void*>(mixk), (int)lds)) return DCHAG_ERR_LAUNCH;
  StageTimer tm(DCHAG_STAGE_TOKENIZE_MIX, st);
  mixk<<<dim3((unsigned)(((N + PB - 1) / PB) * (D / 256)), G, B), wide ? 512 : 256, lds, st>>>(
      C, H, W, p, D, g, static_cast<const bf16*>(x), static_cast<const bf16*>(We), static_cast<const bf16*>(be),
      static_cast<const bf16*>(ce), static_cast<const bf16*>(lv->Wv), static_cast<const bf16*>(lv->bv), y);
  return launch_status();
}

#include "host_train.h"

}  // namespace

// Device address of `scratch` on the current device, looked up once per device (each device holds its own copy of
// the array at its own address).
static int static_scratch(unsigned char** out) {
  static std::mutex mu;
  static unsigned char* ptr[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DCHAG_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DCHAG_ERR_LAUNCH;
    ptr[dev] = static_cast<unsigned char*>(p);
  }
  *out = ptr[dev];
  return DCHAG_OK;
}

extern "C" {

const char* dchag_version(void) { return "0.3"; }

void dchag_debug_reload(void) { g_switches.read(); }

int dchag_profile_begin(void) {
  for (StageRecord& r : g_records) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_records.clear();
  g_profiling = true;
  return DCHAG_OK;
}

int dchag_profile_end(dchag_stage_time* records, int cap) {
  g_profiling = false;
  int n = 0, rc = DCHAG_OK;
  for (StageRecord& r : g_records) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
      rc = DCHAG_ERR_LAUNCH;
    if (records && n < cap) {
      records[n].stage = r.stage;
      records[n].level = r.level;
      records[n].ms = ms;
    }
    ++n;
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_records.clear();
  return rc ? rc : n;
}

int dchag_yardstick_mfma(int iters, float* sink, size_t sink_floats, double* flops, void* stream) {
  if (!sink || !flops) return DCHAG_ERR_NULL;
  if (iters < 1) return DCHAG_ERR_SHAPE;
  if (misaligned(sink)) return DCHAG_ERR_ALIGN;
  const int blocks = 4 * compute_units();                 // 16 wavefronts per compute unit, four per SIMD
  if (sink_floats < (size_t)blocks * 256) return DCHAG_ERR_WORKSPACE;
  k_yardstick_mfma<<<dim3(blocks), 256, 0, static_cast<hipStream_t>(stream)>>>(iters, sink);
  *flops = (double)blocks * 4.0 * (double)iters * 8.0 * 32768.0;
  return launch_status();
}

int dchag_yardstick_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return DCHAG_ERR_NULL;
  if (bytes == 0 || bytes % 16) return DCHAG_ERR_SHAPE;
  if (misaligned(dst) || misaligned(src)) return DCHAG_ERR_ALIGN;
  const size_t pieces = bytes / 16, blocks = (pieces + 1023) / 1024;
  if (blocks > 0x7fffffffu) return DCHAG_ERR_SHAPE;
  k_yardstick_copy<<<dim3((unsigned)blocks), 256, 0, static_cast<hipStream_t>(stream)>>>(
      pieces, static_cast<const f32x4*>(src), static_cast<f32x4*>(dst));
  return launch_status();
}

int dchag_yardstick_read(const void* src, size_t bytes, float* sink, void* stream) {
  if (!src || !sink) return DCHAG_ERR_NULL;
  if (bytes == 0 || bytes % 16) return DCHAG_ERR_SHAPE;
  if (misaligned(src) || misaligned(sink)) return DCHAG_ERR_ALIGN;
  const size_t pieces = bytes / 16, blocks = (pieces + 1023) / 1024;
  if (blocks > 0x7fffffffu) return DCHAG_ERR_SHAPE;
  k_yardstick_read<<<dim3((unsigned)blocks), 256, 0, static_cast<hipStream_t>(stream)>>>(
      pieces, static_cast<const f32x4*>(src), sink);
  return launch_status();
}

const char* dchag_strerror(int status) {
  switch (status) {
    case DCHAG_OK: return "ok";
    case DCHAG_ERR_NULL: return "a required pointer is NULL";
    case DCHAG_ERR_SHAPE: return "sizes do not fit together";
    case DCHAG_ERR_DTYPE: return "unknown dtype";
    case DCHAG_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case DCHAG_ERR_LAUNCH: return "kernel launch failed";
    case DCHAG_ERR_ALIGN: return "a tensor pointer is not 16-byte aligned";
    default: return "unknown status";
  }
}

size_t dchag_workspace_bytes(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, int n_levels,
                             const int32_t* group_sizes, int which) {
  if (dt != DCHAG_F32 && dt != DCHAG_BF16) return 0;
  if (!group_sizes || n_levels < 1 || p < 1 || H < 1 || W < 1 || H % p || W % p) return 0;
  const int N = (H / p) * (W / p);
  if (check_level_shape(B, C, N, D, heads, group_sizes[0]) != DCHAG_OK) return 0;
  if (which == 0) return level_ws(dt, B, C, N, D, heads, group_sizes[0]).total;
  if (which == 1) return forward_ws(dt, B, C, N, p * p, D, heads, n_levels, group_sizes).total;
  if (n_levels > 16) return 0;
  if (which == 2) return folded_ws(dt, B, C, N, p * p, D, heads, n_levels, group_sizes).total;
  if (which == 3) return backward_ws(dt, B, C, N, p * p, D, heads, n_levels, group_sizes, nullptr).total;
  return 0;
}

int dchag_tokenize(dchag_dtype dt, int B, int C, int H, int W, int p, int D, const void* x, const void* We,
                   const void* be, const void* ce, void* tokens, void* stream) {
  if (dt != DCHAG_F32 && dt != DCHAG_BF16) return DCHAG_ERR_DTYPE;
  if (!x || !We || !tokens) return DCHAG_ERR_NULL;
  int rc = check_tokenize_shape(B, C, H, W, p, D);
  if (rc) return rc;
  if (misaligned(x) || misaligned(We) || misaligned(be) || misaligned(ce) || misaligned(tokens)) return DCHAG_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dt == DCHAG_F32)
    return launch_tokenize<float>(B, C, H, W, p, D, static_cast<const float*>(x), static_cast<const float*>(We),
                                  static_cast<const float*>(be), static_cast<const float*>(ce),
                                  static_cast<float*>(tokens), st);
  if ((p * p) % 16 == 0 && p * p <= 256 && D % 64 == 0 && !dbg(SW_GENERIC_TOKENIZE))
    return launch_tokenize_mfma(B, C, H, W, p, D, static_cast<const bf16*>(x), static_cast<const bf16*>(We),
                                static_cast<const bf16*>(be), static_cast<const bf16*>(ce),
                                static_cast<bf16*>(tokens), st);
  return launch_tokenize<bf16>(B, C, H, W, p, D, static_cast<const bf16*>(x), static_cast<const bf16*>(We),
                               static_cast<const bf16*>(be), static_cast<const bf16*>(ce),
                               static_cast<bf16*>(tokens), st);
}

int dchag_aggregate_level(dchag_dtype dt, int B, int Cin, int N, int D, int heads, const dchag_level* lvl,
                          const void* tokens_in, void* tokens_out, void* workspace, size_t workspace_bytes,
                          void* stream) {
  if (dt != DCHAG_F32 && dt != DCHAG_BF16) return DCHAG_ERR_DTYPE;
  if (!tokens_in || !tokens_out) return DCHAG_ERR_NULL;
  int rc = check_level(lvl);
  if (rc) return rc;
  if ((rc = check_level_shape(B, Cin, N, D, heads, lvl->group_size))) return rc;
  if (misaligned(tokens_in) || misaligned(tokens_out)) return DCHAG_ERR_ALIGN;
  if (lvl->kind == DCHAG_LEVEL_LINEAR) {  // needs no workspace
    set_level(1);
    if (dt == DCHAG_F32)
      return run_level_linear<float>(B, Cin, N, D, lvl, static_cast<const float*>(tokens_in),
                                     static_cast<float*>(tokens_out), static_cast<hipStream_t>(stream));
    return run_level_linear<bf16>(B, Cin, N, D, lvl, static_cast<const bf16*>(tokens_in),
                                  static_cast<bf16*>(tokens_out), static_cast<hipStream_t>(stream));
  }
  const size_t need = level_ws(dt, B, Cin, N, D, heads, lvl->group_size).total;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) || workspace_bytes < need)
    return DCHAG_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  set_level(1);
  if (dt == DCHAG_F32)
    return run_level<float>(dt, B, Cin, N, D, heads, lvl, static_cast<const float*>(tokens_in),
                            static_cast<float*>(tokens_out), ws, st);
  if (fast_level(dt, D, heads) && !dbg(SW_GENERIC_LEVEL))
    return run_level_fast(B, Cin, N, D, heads, lvl, static_cast<const bf16*>(tokens_in),
                          static_cast<bf16*>(tokens_out), ws, st);
  return run_level<bf16>(dt, B, Cin, N, D, heads, lvl, static_cast<const bf16*>(tokens_in),
                         static_cast<bf16*>(tokens_out), ws, st);
}

int dchag_aggregate_level_static(dchag_dtype dt, int B, int Cin, int N, int D, int heads, const dchag_level* lvl,
                                 const void* tokens_in, void* tokens_out, void* stream) {
  if (dt != DCHAG_F32 && dt != DCHAG_BF16) return DCHAG_ERR_DTYPE;
  if (!tokens_in || !tokens_out) return DCHAG_ERR_NULL;
  int rc = check_level(lvl);
  if (rc) return rc;
  if ((rc = check_level_shape(B, Cin, N, D, heads, lvl->group_size))) return rc;
  // the size check comes before the first touch of the device, so an oversized call never costs a symbol lookup
  if (lvl->kind != DCHAG_LEVEL_LINEAR &&
      level_ws(dt, B, Cin, N, D, heads, lvl->group_size).total > (size_t)DCHAG_STATIC_SCRATCH_BYTES)
    return DCHAG_ERR_WORKSPACE;
  unsigned char* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  return dchag_aggregate_level(dt, B, Cin, N, D, heads, lvl, tokens_in, tokens_out, ws, DCHAG_STATIC_SCRATCH_BYTES,
                               stream);
}

// dchag_forward and dchag_forward_pos: pos (or NULL) is added to the output in the epilogue of the last level's
// output projection.
static int forward_impl(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                        const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                        const void* pos, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  if (dt != DCHAG_F32 && dt != DCHAG_BF16) return DCHAG_ERR_DTYPE;
  if (!x || !We || !out || !levels) return DCHAG_ERR_NULL;
  if (n_levels < 1 || n_levels > 16) return DCHAG_ERR_SHAPE;
  int rc = check_tokenize_shape(B, C, H, W, p, D);
  if (rc) return rc;
  const int N = (H / p) * (W / p);
  int32_t gs[16];
  int c_in = C;
  for (int l = 0; l < n_levels; ++l) {
    if ((rc = check_level(&levels[l]))) return rc;
    if ((rc = check_level_shape(B, c_in, N, D, heads, levels[l].group_size))) return rc;
    gs[l] = levels[l].group_size;
    c_in = groups_of(c_in, gs[l]);
  }
  if (c_in != 1 || levels[n_levels - 1].kind != DCHAG_LEVEL_ATTENTION) return DCHAG_ERR_SHAPE;
  if (misaligned(x) || misaligned(We) || misaligned(be) || misaligned(ce) || misaligned(out) || misaligned(pos))
    return DCHAG_ERR_ALIGN;
  const ForwardWs w = forward_ws(dt, B, C, N, p * p, D, heads, n_levels, gs);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) || w.total == 0 ||
      workspace_bytes < w.total)
    return DCHAG_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);

  set_level(0);
  const void* zin = ws + w.tokens;
  c_in = C;
  int first = 0;
  const int pp0 = p * p;
  if (tokenize_mix_ok(dt, levels, pp0, D)) {
    set_level(1);
    bf16* y = reinterpret_cast<bf16*>(ws + w.ping);
    if ((rc = tokenize_mix_forward(B, C, H, W, p, D, x, We, be, ce, &levels[0], y, st))) return rc;
    zin = y;
    c_in = groups_of(C, gs[0]);
    first = 1;
  } else if ((rc = dchag_tokenize(dt, B, C, H, W, p, D, x, We, be, ce, ws + w.tokens, stream)))
    return rc;
  // every attention level's weight-only prep (projected query, query folded into the key weights) in ONE launch
  const bool fast = dt == DCHAG_BF16 && fast_level(dt, D, heads) && !dbg(SW_GENERIC_LEVEL);
  PrepBufs ready[16];
  if (fast) {
    KeyPrepJob jobs[16];
    int nj = 0, cl = c_in;
    for (int l = first; l < n_levels; ++l) {
      const int G = groups_of(cl, gs[l]);
      if (levels[l].kind == DCHAG_LEVEL_ATTENTION) {
        ready[l] = prep_bufs(ws + w.prep[l], G, D, heads);
        const bool px0 = l == 0 && pixel_scores_ok(p, heads);
        jobs[nj++] = KeyPrepJob{&levels[l], G, ready[l], px0 ? reinterpret_cast<float*>(ws + w.mft) : nullptr};
      }
      cl = G;
    }
    set_level(0);
    if (nj && (rc = launch_query_keys(D, heads, jobs, nj, st))) return rc;
  }
  for (int l = first; l < n_levels; ++l) {
    set_level(l + 1);
    void* zout = (l + 1 == n_levels) ? out : static_cast<void*>(ws + ((l & 1) ? w.pong : w.ping));
    const void* rowadd = (l + 1 == n_levels) ? pos : nullptr;
    if (levels[l].kind == DCHAG_LEVEL_LINEAR)
      rc = (dt == DCHAG_F32) ? run_level_linear<float>(B, c_in, N, D, &levels[l], static_cast<const float*>(zin),
                                                       static_cast<float*>(zout), st)
                             : run_level_linear<bf16>(B, c_in, N, D, &levels[l], static_cast<const bf16*>(zin),
                                                      static_cast<bf16*>(zout), st);
    else if (dt == DCHAG_F32)
      rc = run_level<float>(dt, B, c_in, N, D, heads, &levels[l], static_cast<const float*>(zin),
                            static_cast<float*>(zout), ws + w.level, st, static_cast<const float*>(rowadd));
    else if (fast_level(dt, D, heads) && !dbg(SW_GENERIC_LEVEL)) {
      PixelScores px{static_cast<const bf16*>(x), static_cast<const bf16*>(We), static_cast<const bf16*>(be),
                     static_cast<const bf16*>(ce), H, W, p, reinterpret_cast<float*>(ws + w.ms),
                     reinterpret_cast<float*>(ws + w.cs), reinterpret_cast<float*>(ws + w.mft),
                     reinterpret_cast<bf16*>(ws + w.msb)};
      const bool use_px = (l == 0) && pixel_scores_ok(p, heads);
      rc = run_level_fast(B, c_in, N, D, heads, &levels[l], static_cast<const bf16*>(zin),
                          static_cast<bf16*>(zout), ws + w.level, st, use_px ? &px : nullptr,
                          static_cast<const bf16*>(rowadd), &ready[l]);
    }
    else
      rc = run_level<bf16>(dt, B, c_in, N, D, heads, &levels[l], static_cast<const bf16*>(zin),
                           static_cast<bf16*>(zout), ws + w.level, st, static_cast<const bf16*>(rowadd));
    if (rc) return rc;
    zin = zout;
    c_in = groups_of(c_in, gs[l]);
  }
  return DCHAG_OK;
}

int dchag_forward(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                  const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                  void* out, void* workspace, size_t workspace_bytes, void* stream) {
  return forward_impl(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, nullptr, out, workspace,
                      workspace_bytes, stream);
}

int dchag_forward_pos(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                      const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                      const void* pos, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!pos) return DCHAG_ERR_NULL;
  return forward_impl(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, pos, out, workspace,
                      workspace_bytes, stream);
}

// Shared argument checks of the calls that take the whole chain of levels; fills gs / kinds.
static int check_chain(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                       const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                       int32_t* gs, int32_t* kinds) {
  if (dt != DCHAG_F32 && dt != DCHAG_BF16) return DCHAG_ERR_DTYPE;
  if (!x || !We || !levels) return DCHAG_ERR_NULL;
  if (n_levels < 1 || n_levels > 16) return DCHAG_ERR_SHAPE;
  int rc = check_tokenize_shape(B, C, H, W, p, D);
  if (rc) return rc;
  const int N = (H / p) * (W / p);
  int c_in = C;
  for (int l = 0; l < n_levels; ++l) {
    if ((rc = check_level(&levels[l]))) return rc;
    if ((rc = check_level_shape(B, c_in, N, D, heads, levels[l].group_size))) return rc;
    gs[l] = levels[l].group_size;
    kinds[l] = levels[l].kind;
    c_in = groups_of(c_in, gs[l]);
  }
  if (c_in != 1 || levels[n_levels - 1].kind != DCHAG_LEVEL_ATTENTION) return DCHAG_ERR_SHAPE;
  if (misaligned(x) || misaligned(We) || misaligned(be) || misaligned(ce)) return DCHAG_ERR_ALIGN;
  return DCHAG_OK;
}

int dchag_forward_folded(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                         const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                         void* out, void* workspace, size_t workspace_bytes, void* stream) {
  int32_t gs[16], kinds[16];
  int rc = check_chain(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, kinds);
  if (rc) return rc;
  if (!out) return DCHAG_ERR_NULL;
  if (misaligned(out)) return DCHAG_ERR_ALIGN;
  const int N = (H / p) * (W / p);
  const FoldedWs w = folded_ws(dt, B, C, N, p * p, D, heads, n_levels, gs);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) || w.total == 0 ||
      workspace_bytes < w.total)
    return DCHAG_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  if (dt == DCHAG_F32)
    return forward_folded_impl<float>(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, out, ws, w, st);
  return forward_folded_impl<bf16>(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, out, ws, w, st);
}

// Shared checks of the two calls that size and fill a prepared buffer: the chain of levels and its first level's route.
static int check_prepare(dchag_dtype dt, int C, int p, int D, int heads, int n_levels, const dchag_level* levels) {
  if (dt != DCHAG_F32 && dt != DCHAG_BF16) return DCHAG_ERR_DTYPE;
  if (!levels) return DCHAG_ERR_NULL;
  if (n_levels < 1 || n_levels > 16 || C < 1 || p < 1 || p > 64 || D < 1 || heads < 1 || D % heads ||
      (long)C * D * p * p > (1L << 40))
    return DCHAG_ERR_SHAPE;
  int c_in = C;
  for (int l = 0; l < n_levels; ++l) {
    if (levels[l].group_size < 1 || (levels[l].kind != DCHAG_LEVEL_ATTENTION && levels[l].kind != DCHAG_LEVEL_LINEAR))
      return DCHAG_ERR_SHAPE;
    c_in = groups_of(c_in, levels[l].group_size);
  }
  if (c_in != 1 || levels[n_levels - 1].kind != DCHAG_LEVEL_ATTENTION) return DCHAG_ERR_SHAPE;
  return values_from_pixels(dt, p, D, heads, &levels[0]) ? DCHAG_OK : DCHAG_ERR_SHAPE;
}

size_t dchag_value_fold_bytes(dchag_dtype dt, int C, int p, int D, int heads, int n_levels, const dchag_level* levels) {
  if (check_prepare(dt, C, p, D, heads, n_levels, levels)) return 0;
  return prepared_layout(C, p * p, D, heads, n_levels, levels).total;
}

int dchag_fold_value(dchag_dtype dt, int C, int p, int D, int heads, const void* We, const void* be, const void* ce,
                     int n_levels, const dchag_level* levels, void* folded, size_t folded_bytes, void* stream) {
  int rc = check_prepare(dt, C, p, D, heads, n_levels, levels);
  if (rc) return rc;                                     // DCHAG_ERR_SHAPE: nothing to prepare for this shape
  if (!We || !folded) return DCHAG_ERR_NULL;
  for (int l = 0; l < n_levels; ++l)
    if ((rc = check_level(&levels[l]))) return rc;
  if (misaligned(We) || misaligned(be) || misaligned(ce)) return DCHAG_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(folded) & (kAlign - 1)) ||
      folded_bytes < prepared_layout(C, p * p, D, heads, n_levels, levels).total)
    return DCHAG_ERR_WORKSPACE;
  // the patch size stands in for the image size: the prep reads weights only
  return prepare_folded(C, p, p, p, D, heads, We, be, ce, n_levels, levels, static_cast<unsigned char*>(folded),
                        static_cast<hipStream_t>(stream));
}

int dchag_forward_prefolded(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                            const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                            const void* folded, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  int32_t gs[16], kinds[16];
  int rc = check_chain(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, kinds);
  if (rc) return rc;
  if (!out || !folded) return DCHAG_ERR_NULL;
  if (misaligned(out)) return DCHAG_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(folded) & (kAlign - 1)) return DCHAG_ERR_WORKSPACE;
  if (!values_from_pixels(dt, p, D, heads, &levels[0])) return DCHAG_ERR_SHAPE;
  const int N = (H / p) * (W / p);
  const FoldedWs w = folded_ws(dt, B, C, N, p * p, D, heads, n_levels, gs);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) || w.total == 0 ||
      workspace_bytes < w.total)
    return DCHAG_ERR_WORKSPACE;
  return forward_folded_impl<bf16>(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, out,
                                   static_cast<unsigned char*>(workspace), w, static_cast<hipStream_t>(stream),
                                   static_cast<const unsigned char*>(folded));
}

// which: 1 = forward that keeps, 2 = reverse sweep, 3 = both (dchag_backward)
static int train_call(int which, dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                      const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels, void* out,
                      const void* dout, void* dx, void* dWe, void* dtok_bias, const dchag_level_grads* grads,
                      void* workspace, size_t workspace_bytes, void* stream) {
  int32_t gs[16], kinds[16];
  int rc = check_chain(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, kinds);
  if (rc) return rc;
  if ((which & 2) && (!dout || !grads)) return DCHAG_ERR_NULL;
  if (which == 1 && !out) return DCHAG_ERR_NULL;
  if (misaligned(out) || misaligned(dout) || misaligned(dx) || misaligned(dWe) || misaligned(dtok_bias))
    return DCHAG_ERR_ALIGN;
  if (which & 2)
    for (int l = 0; l < n_levels; ++l) {
      const void* ps[] = {grads[l].dquery, grads[l].dWq, grads[l].dWk, grads[l].dWv, grads[l].dWo,
                          grads[l].dbq,    grads[l].dbk, grads[l].dbv, grads[l].dbo};
      for (const void* q : ps)
        if (misaligned(q)) return DCHAG_ERR_ALIGN;
    }
  const int N = (H / p) * (W / p);
  const BackwardWs w = backward_ws(dt, B, C, N, p * p, D, heads, n_levels, gs, kinds);
  // a keep / reverse pair shares one workspace, so both are held to the size dchag_workspace_bytes reports
  const size_t need = which == 3 ? w.total : backward_ws(dt, B, C, N, p * p, D, heads, n_levels, gs, nullptr).total;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) || w.total == 0 || workspace_bytes < need)
    return DCHAG_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  if (which & 1) {
    rc = dt == DCHAG_F32 ? keep_forward<float>(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, out, ws, w, st)
                         : keep_forward<bf16>(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, out, ws, w, st);
    if (rc) return rc;
  }
  if (which & 2)
    rc = dt == DCHAG_F32 ? reverse_sweep<float>(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, dout, dx, dWe,
                                                dtok_bias, grads, ws, w, st)
                         : reverse_sweep<bf16>(dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, gs, dout, dx, dWe,
                                               dtok_bias, grads, ws, w, st);
  return rc;
}

int dchag_backward(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                   const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                   const void* dout, void* dx, void* dWe, void* dtok_bias, const dchag_level_grads* grads,
                   void* workspace, size_t workspace_bytes, void* stream) {
  return train_call(3, dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, nullptr, dout, dx, dWe, dtok_bias,
                    grads, workspace, workspace_bytes, stream);
}

int dchag_forward_keep(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                       const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                       void* out, void* workspace, size_t workspace_bytes, void* stream) {
  return train_call(1, dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, out, nullptr, nullptr, nullptr,
                    nullptr, nullptr, workspace, workspace_bytes, stream);
}

int dchag_backward_kept(dchag_dtype dt, int B, int C, int H, int W, int p, int D, int heads, const void* x,
                        const void* We, const void* be, const void* ce, int n_levels, const dchag_level* levels,
                        const void* dout, void* dx, void* dWe, void* dtok_bias, const dchag_level_grads* grads,
                        void* workspace, size_t workspace_bytes, void* stream) {
  return train_call(2, dt, B, C, H, W, p, D, heads, x, We, be, ce, n_levels, levels, nullptr, dout, dx, dWe, dtok_bias,
                    grads, workspace, workspace_bytes, stream);
}

}  // extern "C"
