// Host side of libqaq: argument checking, cache bookkeeping, thresholds, launches.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "qaq_internal.h"

struct qaq_cache {
  qaq_config cfg;
  std::vector<float> qnorm2;
  std::vector<float> othr;
  QaqDims dims;
  QaqArena arena;
  QaqView view;
  int len;                         // cached positions of the longest sequence
  int max_shortfall;               // 0: every sequence has `len` positions; else sequence b has max(len - view.shortfall[b], 0)
  int n_o;
  int ring_next;                   // ring row that the next score row goes to
  int update_parity;               // which of the two hand-over counters the next decode-step update uses
  int row_len[QAQ_MAX_WINDOW];     // tokens covered by each ring row (0 = empty)
  double sigma_s, sigma_x;
  std::vector<hipEvent_t> prof_ev;  // 4 events per profiled attention call
  int prof_n;
  std::vector<int> prof_kernels;    // dispatches each profiled call made
};

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(QAQ_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

int outliers_per_side(const qaq_config* cfg) {
  if (cfg->n_outlier_per_side >= 0) return cfg->n_outlier_per_side;
  if (!(cfg->outlier_frac > 0.0f)) return 0;
  return (int)std::ceil((double)cfg->outlier_frac / 2.0 * cfg->head_dim - 1e-12);
}

bool valid_config(const qaq_config* c, QaqDims* d) {
  if (!c) { fail(QAQ_ERR_INVALID_ARG, "config is NULL"); return false; }
  if (c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads) {
    fail(QAQ_ERR_INVALID_ARG, "bad batch/head counts (%d, %d, %d)", c->batch, c->n_q_heads, c->n_kv_heads); return false; }
  if (c->n_kv_heads > QAQ_MAX_KV_HEADS) { fail(QAQ_ERR_INVALID_ARG, "at most %d KV heads", QAQ_MAX_KV_HEADS); return false; }
  if (c->head_dim != 64 && c->head_dim != 128) { fail(QAQ_ERR_INVALID_ARG, "head_dim must be 64 or 128, got %d", c->head_dim); return false; }
  if (c->max_tokens < 1) { fail(QAQ_ERR_INVALID_ARG, "max_tokens must be positive"); return false; }
  if (c->n_bits < 1 || c->n_bits > 5) { fail(QAQ_ERR_INVALID_ARG, "n_bits must be 1..5"); return false; }
  for (int i = 0; i < c->n_bits; ++i) {
    const int b = c->bit_set[i];
    if (!(b == 1 || b == 2 || b == 3 || b == 4 || b == 8) || (i && b <= c->bit_set[i - 1])) {
      fail(QAQ_ERR_INVALID_ARG, "bit_set must be an ascending subset of {1,2,3,4,8}"); return false; }
  }
  if (c->window < 1 || c->window > QAQ_MAX_WINDOW) { fail(QAQ_ERR_INVALID_ARG, "window must be 1..%d", QAQ_MAX_WINDOW); return false; }
  const int no = outliers_per_side(c);
  if (no < 0 || 2 * no > QAQ_MAX_NO2 || c->head_dim - 2 * no < 2) { fail(QAQ_ERR_INVALID_ARG, "unsupported outlier count %d per side", no); return false; }
  if (!(c->sigma_s_max > 0.0) || !(c->sigma_x_max > 0.0)) { fail(QAQ_ERR_INVALID_ARG, "sigma bounds must be positive"); return false; }
  if (!c->qnorm2) { fail(QAQ_ERR_INVALID_ARG, "qnorm2 is NULL"); return false; }
  for (int h = 0; h < c->n_kv_heads; ++h)
    if (!(c->qnorm2[h] > 0.0f)) { fail(QAQ_ERR_INVALID_ARG, "qnorm2[%d] must be positive", h); return false; }
  d->B = c->batch; d->Hq = c->n_q_heads; d->Hkv = c->n_kv_heads; d->D = c->head_dim;
  d->NT = (c->max_tokens + QAQ_TT - 1) / QAQ_TT;
  d->Tmax = d->NT * QAQ_TT;
  d->no2 = 2 * no;
  d->window = c->window;
  if (c->window_store < QAQ_WINDOW_FP32 || c->window_store > QAQ_WINDOW_BF16) { fail(QAQ_ERR_INVALID_ARG, "window_store must be 0 (fp32), 1 (fp16) or 2 (bf16)"); return false; }
  d->ring_half = c->window_store;
  d->csr = c->outlier_thresholds != nullptr;
  if (d->csr) {
    if (no < 1) { fail(QAQ_ERR_INVALID_ARG, "outlier thresholds need a cap of 1..4 outliers per end"); return false; }
    for (int i = 0; i < 2 * c->n_kv_heads; ++i)
      if (!(c->outlier_thresholds[2 * i] <= c->outlier_thresholds[2 * i + 1])) {
        fail(QAQ_ERR_INVALID_ARG, "outlier thresholds must satisfy lo <= hi"); return false; }
  }
  return true;
}

void thresholds(const qaq_cache* c, int T, float* tau_k, float* c_v) {
  for (int h = 0; h < c->dims.Hkv; ++h) {
    if (T < 2) { tau_k[h] = INFINITY; continue; }
    const double var_k = std::log1p((double)T * T * T / (T - 1.0) * c->sigma_s * c->sigma_s) / (double)c->qnorm2[h];
    tau_k[h] = (float)(2.0 * std::sqrt(3.0) * std::sqrt(var_k));
  }
  *c_v = (float)(2.0 * std::sqrt(3.0) * c->sigma_x / std::sqrt((double)(T < 1 ? 1 : T)));
}

int seq_len(const qaq_cache* c, int b, int len_longest) {
  const int l = len_longest - (c->max_shortfall ? c->view.shortfall[b] : 0);
  return l > 0 ? l : 0;
}

// The tables a kernel call gets: thresholds for T tokens in the longest sequence -- per KV head, or,
// where lengths differ, per (sequence, KV head) for the key rule and per sequence for the value rule,
// each from the sequence's own token count.
void threshold_tables(const qaq_cache* c, int T, float* tau_k, float* c_v) {
  if (!c->max_shortfall) { thresholds(c, T, tau_k, c_v); return; }
  for (int b = 0; b < c->dims.B; ++b) thresholds(c, seq_len(c, b, T), tau_k + (size_t)b * c->dims.Hkv, c_v + b);
}

// first tile that holds the position after the end of any sequence
int first_open_tile(const qaq_cache* c) {
  const int shortest = c->len - c->max_shortfall;
  return (shortest > 0 ? shortest : 0) / QAQ_TT;
}

// on an empty cache whose sequences differ in length, the first append must give every sequence a token
bool first_append_too_short(const qaq_cache* c, int n_new) {
  if (c->len == 0 && c->max_shortfall >= n_new) {
    fail(QAQ_ERR_INVALID_ARG, "the first append of %d tokens leaves the sequence that is %d tokens shorter empty", n_new, c->max_shortfall);
    return true;
  }
  return false;
}

}  // namespace

// ---- streaming yardsticks ------------------------------------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Every workgroup walks over contiguous 16 KB blocks (four 16-byte loads per thread in
// flight) and folds what it read into one word so that the compiler keeps the loads.
__global__ void __launch_bounds__(256) k_stream_read(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
  u32x4 acc = {0, 0, 0, 0};
  const size_t nblk = n16 / 1024;                       // whole blocks of 1024 x 16 bytes
  for (size_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
    const u32x4* p = src + blk * 1024 + threadIdx.x;
    const u32x4 a = __builtin_nontemporal_load(p), b = __builtin_nontemporal_load(p + 256);
    const u32x4 c = __builtin_nontemporal_load(p + 512), d = __builtin_nontemporal_load(p + 768);
    acc ^= a ^ b ^ c ^ d;
  }
  for (size_t i = nblk * 1024 + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256)
    acc ^= __builtin_nontemporal_load(src + i);
  uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
  for (int o = 32; o; o >>= 1) x ^= __shfl_xor(x, o);
  __shared__ uint32_t part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = x;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

__global__ void __launch_bounds__(256) k_stream_copy(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16) {
  size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

extern "C" {

const char* qaq_last_error(void) { return g_err; }

int qaq_outliers_per_side(const qaq_config* cfg) {
  QaqDims d;
  if (!valid_config(cfg, &d)) return QAQ_ERR_INVALID_ARG;
  return d.no2 / 2;
}

size_t qaq_arena_bytes(const qaq_config* cfg) {
  QaqDims d;
  if (!valid_config(cfg, &d)) return 0;
  return qaq_carve(d).total;
}

int qaq_create(const qaq_config* cfg, void* dev_arena, size_t arena_bytes, qaq_cache** out) {
  QaqDims d;
  if (!out) return fail(QAQ_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  if (!valid_config(cfg, &d)) return QAQ_ERR_INVALID_ARG;
  if (!dev_arena || ((uintptr_t)dev_arena & 255)) return fail(QAQ_ERR_INVALID_ARG, "arena must be non-NULL and 256-byte aligned");
  const QaqArena a = qaq_carve(d);
  if (arena_bytes < a.total) return fail(QAQ_ERR_CAPACITY, "arena has %zu bytes, %zu needed", arena_bytes, a.total);
  qaq_cache* c = new (std::nothrow) qaq_cache();
  if (!c) return fail(QAQ_ERR_INVALID_ARG, "out of host memory");
  c->cfg = *cfg;
  c->qnorm2.assign(cfg->qnorm2, cfg->qnorm2 + cfg->n_kv_heads);
  c->cfg.qnorm2 = c->qnorm2.data();
  if (d.csr) {
    c->othr.assign(cfg->outlier_thresholds, cfg->outlier_thresholds + 4 * cfg->n_kv_heads);
    c->cfg.outlier_thresholds = c->othr.data();
  }
  c->dims = d;
  c->arena = a;
  c->n_o = d.no2 / 2;
  c->len = 0;
  c->max_shortfall = 0;
  c->ring_next = 0;
  c->update_parity = 0;
  std::memset(c->row_len, 0, sizeof(c->row_len));
  c->sigma_s = cfg->sigma_s_max;
  c->sigma_x = cfg->sigma_x_max;
  c->prof_n = 0;
  uint8_t* base = (uint8_t*)dev_arena;
  QaqView& v = c->view;
  for (int s = 0; s < 2; ++s) {
    v.codes[s] = base + a.codes[s];
    v.mm[s] = (uint32_t*)(base + a.mm[s]);
    v.perm[s] = base + a.perm[s];
    v.oidx[s] = base + a.oidx[s];
    v.oval[s] = (uint16_t*)(base + a.oval[s]);
    v.tags[s] = base + a.tags[s];
  }
  v.counts = (uint16_t*)(base + a.counts);
  v.vbound = (float*)(base + a.vbound);
  v.kthr = (float*)(base + a.kthr);
  v.ring = base + a.ring;
  v.ring_half = d.ring_half;
  v.partial = (float*)(base + a.partial);
  v.statbuf = (long long*)(base + a.statbuf);
  v.refused = (unsigned int*)(base + a.refused);
  v.todo = (uint32_t*)(base + a.todo);
  v.todo_count = (uint32_t*)(base + a.todo_count);
  v.B = d.B; v.Hq = d.Hq; v.Hkv = d.Hkv; v.D = d.D; v.Tmax = d.Tmax; v.NT = d.NT; v.no2 = d.no2; v.window = d.window;
  v.has1 = cfg->bit_set[0] == 1;
  v.csr = d.csr;
  v.ragged = 0;
  std::memset(v.shortfall, 0, sizeof(v.shortfall));
  for (int s = 0; s < 2; ++s) {
    v.ostart[s] = d.csr ? (uint16_t*)(base + a.ostart[s]) : nullptr;
    v.ocnt[s] = d.csr ? base + a.ocnt[s] : nullptr;
  }
  v.othr = d.csr ? (const float*)(base + a.othr) : nullptr;
  if (d.csr) {
    hipError_t e0 = hipMemcpy(base + a.othr, c->othr.data(), c->othr.size() * sizeof(float), hipMemcpyHostToDevice);
    if (e0 != hipSuccess) { delete c; return hip_fail(e0, "qaq_create: thresholds"); }
  }
  v.cap[0] = qaq_k_cap(d.D);
  v.cap[1] = qaq_v_cap(d.D);
  hipError_t e = qaq_launch_init(v, nullptr);
  if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
  if (e != hipSuccess) { delete c; return hip_fail(e, "qaq_create: init"); }
  *out = c;
  return QAQ_OK;
}

int qaq_destroy(qaq_cache* c) {
  if (c) for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  delete c;
  return QAQ_OK;
}

int qaq_reset(qaq_cache* c) {
  if (!c) return fail(QAQ_ERR_INVALID_ARG, "cache is NULL");
  c->len = 0;
  c->max_shortfall = 0;
  c->view.ragged = 0;
  std::memset(c->view.shortfall, 0, sizeof(c->view.shortfall));
  c->ring_next = 0;
  std::memset(c->row_len, 0, sizeof(c->row_len));
  return QAQ_OK;
}

int qaq_length(const qaq_cache* c, int32_t* host_len) {
  if (!c || !host_len) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  *host_len = c->len;
  return QAQ_OK;
}

int qaq_lengths(const qaq_cache* c, int32_t* host_len) {
  if (!c || !host_len) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  for (int b = 0; b < c->dims.B; ++b) host_len[b] = seq_len(c, b, c->len);
  return QAQ_OK;
}

int qaq_set_shortfall(qaq_cache* c, const int32_t* host_shortfall) {
  if (!c || !host_shortfall) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  if (c->len != 0) return fail(QAQ_ERR_INVALID_ARG, "the cache already holds %d tokens", c->len);
  for (int r = 0; r < QAQ_MAX_WINDOW; ++r)
    if (c->row_len[r]) return fail(QAQ_ERR_INVALID_ARG, "the attention window already holds score rows");
  int lo = host_shortfall[0], hi = host_shortfall[0];
  for (int b = 1; b < c->dims.B; ++b) { lo = host_shortfall[b] < lo ? host_shortfall[b] : lo; hi = host_shortfall[b] > hi ? host_shortfall[b] : hi; }
  if (lo != 0) return fail(QAQ_ERR_INVALID_ARG, "the smallest shortfall must be 0 (the longest sequence), got %d", lo);
  if (hi >= c->cfg.max_tokens) return fail(QAQ_ERR_CAPACITY, "a shortfall of %d tokens with max_tokens %d", hi, c->cfg.max_tokens);
  if (hi > 0 && (c->dims.B > QAQ_MAX_RAGGED_BATCH || c->dims.B * c->dims.Hkv > QAQ_MAX_THR))
    return fail(QAQ_ERR_INVALID_ARG, "sequences of different lengths: at most %d sequences and %d (sequence, KV head) pairs",
                QAQ_MAX_RAGGED_BATCH, QAQ_MAX_THR);
  c->max_shortfall = hi;
  c->view.ragged = hi > 0;
  std::memset(c->view.shortfall, 0, sizeof(c->view.shortfall));
  if (hi > 0) for (int b = 0; b < c->dims.B; ++b) c->view.shortfall[b] = host_shortfall[b];
  return QAQ_OK;
}

int qaq_set_sigmas(qaq_cache* c, double sigma_s_max, double sigma_x_max) {
  if (!c) return fail(QAQ_ERR_INVALID_ARG, "cache is NULL");
  if (!(sigma_s_max > 0.0) || !(sigma_x_max > 0.0)) return fail(QAQ_ERR_INVALID_ARG, "sigma bounds must be positive");
  c->sigma_s = sigma_s_max;
  c->sigma_x = sigma_x_max;
  return QAQ_OK;
}

int qaq_thresholds(const qaq_cache* c, int32_t T, float* host_tau_k, float* host_c_v) {
  if (!c || !host_tau_k || !host_c_v) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  if (T < 1) return fail(QAQ_ERR_INVALID_ARG, "T must be positive");
  thresholds(c, T, host_tau_k, host_c_v);
  return QAQ_OK;
}

static void fill_bit_set(const qaq_cache* c, QaqRuleArgs& r) {
  r.nbits = c->cfg.n_bits;
  for (int i = 0; i < 5; ++i) r.bit_set[i] = c->cfg.bit_set[i < r.nbits ? i : r.nbits - 1];
}

int qaq_quantize_append(qaq_cache* c, const void* dev_k, const void* dev_v, int32_t n_new,
                        const uint8_t* dev_k_bits, const uint8_t* dev_v_bits, void* stream) {
  if (!c) return fail(QAQ_ERR_INVALID_ARG, "cache is NULL");
  if (n_new < 0) return fail(QAQ_ERR_INVALID_ARG, "n_new is negative");
  if (n_new == 0) return QAQ_OK;
  if (!dev_k || !dev_v) return fail(QAQ_ERR_INVALID_ARG, "K/V input is NULL");
  if (((uintptr_t)dev_k & 15) || ((uintptr_t)dev_v & 15)) return fail(QAQ_ERR_INVALID_ARG, "K/V input must be 16-byte aligned");
  if ((long long)c->len + n_new > c->cfg.max_tokens)
    return fail(QAQ_ERR_CAPACITY, "%d cached + %d new tokens exceed max_tokens %d", c->len, n_new, c->cfg.max_tokens);
  if (first_append_too_short(c, n_new)) return QAQ_ERR_INVALID_ARG;
  QaqBuildArgs a;
  std::memset(&a, 0, sizeof(a));
  a.v = c->view;
  a.mode = 0;
  fill_bit_set(c, a.rule);
  a.len_before = c->len;
  a.len_after = c->len + n_new;
  a.tile0 = first_open_tile(c);
  a.n_new = n_new;
  a.widest = c->cfg.bit_set[c->cfg.n_bits - 1];
  a.newx[0] = (const __half*)dev_k; a.newx[1] = (const __half*)dev_v;
  a.newbits[0] = dev_k_bits; a.newbits[1] = dev_v_bits;
  const int tile_last = (a.len_after - 1) / QAQ_TT;
  hipError_t e = qaq_launch_build(a, tile_last - a.tile0 + 1, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "qaq_quantize_append");
  c->len = a.len_after;
  return QAQ_OK;
}

int qaq_select_bits(qaq_cache* c, const float* dev_scores, uint8_t* dev_k_bits, uint8_t* dev_v_bits, void* stream) {
  if (!c || !dev_k_bits || !dev_v_bits) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  if (c->len == 0) return QAQ_OK;
  QaqSelectArgs a;
  std::memset(&a, 0, sizeof(a));
  a.v = c->view;
  a.len = c->len;
  a.G = c->dims.Hq / c->dims.Hkv;
  a.scores = dev_scores;
  a.new_row = c->ring_next;
  for (int r = 0; r < QAQ_MAX_WINDOW; ++r) a.row_len[r] = r < c->dims.window ? c->row_len[r] : 0;
  if (dev_scores) a.row_len[a.new_row] = c->len;     // the row this call writes (kept by the cache only if the launch succeeds)
  a.nbits = c->cfg.n_bits;
  for (int i = 0; i < 5; ++i) a.bit_set[i] = c->cfg.bit_set[i < a.nbits ? i : a.nbits - 1];
  threshold_tables(c, c->len, a.tau_k, a.c_v);
  a.out_bits[0] = dev_k_bits; a.out_bits[1] = dev_v_bits;
  hipError_t e = qaq_launch_select(a, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "qaq_select_bits");
  if (dev_scores) {
    c->row_len[a.new_row] = c->len;
    c->ring_next = (a.new_row + 1) % c->dims.window;
  }
  return QAQ_OK;
}

int qaq_requantize(qaq_cache* c, const uint8_t* dev_k_bits, const uint8_t* dev_v_bits,
                   const void* dev_k_orig, const void* dev_v_orig, int32_t orig_tokens, void* stream) {
  if (!c) return fail(QAQ_ERR_INVALID_ARG, "cache is NULL");
  if ((dev_k_orig || dev_v_orig) && orig_tokens < c->len)
    return fail(QAQ_ERR_INVALID_ARG, "unquantized copies hold %d tokens, cache has %d", orig_tokens, c->len);
  if (c->len == 0 || (!dev_k_bits && !dev_v_bits)) return QAQ_OK;
  if (((uintptr_t)dev_k_orig & 15) || ((uintptr_t)dev_v_orig & 15)) return fail(QAQ_ERR_INVALID_ARG, "originals must be 16-byte aligned");
  QaqBuildArgs a;
  std::memset(&a, 0, sizeof(a));
  a.v = c->view;
  a.mode = 1;
  fill_bit_set(c, a.rule);
  a.len_before = a.len_after = c->len;
  a.tile0 = 0;
  a.widest = c->cfg.bit_set[c->cfg.n_bits - 1];
  a.newbits[0] = dev_k_bits; a.newbits[1] = dev_v_bits;
  a.orig[0] = (const __half*)dev_k_orig; a.orig[1] = (const __half*)dev_v_orig;
  a.orig_tokens = orig_tokens;
  hipError_t e = qaq_launch_build(a, (c->len + QAQ_TT - 1) / QAQ_TT, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "qaq_requantize");
  return QAQ_OK;
}

int qaq_decode_update(qaq_cache* c, const float* dev_scores, const void* dev_k_new, const void* dev_v_new,
                      void* dev_k_orig, void* dev_v_orig, int32_t orig_tokens,
                      uint8_t* dev_k_bits, uint8_t* dev_v_bits, void* stream) {
  if (!c || !dev_scores || !dev_k_new || !dev_v_new) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  if (((uintptr_t)dev_k_new & 15) || ((uintptr_t)dev_v_new & 15)) return fail(QAQ_ERR_INVALID_ARG, "K/V input must be 16-byte aligned");
  if (((uintptr_t)dev_k_orig & 15) || ((uintptr_t)dev_v_orig & 15)) return fail(QAQ_ERR_INVALID_ARG, "originals must be 16-byte aligned");
  if (c->len + 1 > c->cfg.max_tokens)
    return fail(QAQ_ERR_CAPACITY, "%d cached + 1 new token exceed max_tokens %d", c->len, c->cfg.max_tokens);
  if ((dev_k_orig || dev_v_orig) && orig_tokens < c->len + 1)
    return fail(QAQ_ERR_INVALID_ARG, "unquantized copies hold %d tokens, cache will have %d", orig_tokens, c->len + 1);
  if (first_append_too_short(c, 1)) return QAQ_ERR_INVALID_ARG;
  QaqBuildArgs a;
  std::memset(&a, 0, sizeof(a));
  a.v = c->view;
  a.mode = 2;
  a.len_before = c->len;
  a.len_after = c->len + 1;
  a.tile0 = 0;
  a.n_new = 1;
  a.widest = c->cfg.bit_set[c->cfg.n_bits - 1];
  a.newx[0] = (const __half*)dev_k_new; a.newx[1] = (const __half*)dev_v_new;
  a.orig[0] = (const __half*)dev_k_orig; a.orig[1] = (const __half*)dev_v_orig;
  a.orig_put[0] = (__half*)dev_k_orig; a.orig_put[1] = (__half*)dev_v_orig;
  a.orig_tokens = orig_tokens;
  QaqRuleArgs& r = a.rule;
  r.G = c->dims.Hq / c->dims.Hkv;
  r.scores = dev_scores;
  r.score_stride = a.len_after;
  r.new_row = c->ring_next;
  for (int i = 0; i < QAQ_MAX_WINDOW; ++i) r.row_len[i] = i < c->dims.window ? c->row_len[i] : 0;
  r.row_len[r.new_row] = a.len_after;               // the row this call writes (kept by the cache only if the launch succeeds)
  r.nbits = c->cfg.n_bits;
  for (int i = 0; i < 5; ++i) r.bit_set[i] = c->cfg.bit_set[i < r.nbits ? i : r.nbits - 1];
  threshold_tables(c, a.len_after, r.tau_k, r.c_v);
  r.out_bits[0] = dev_k_bits; r.out_bits[1] = dev_v_bits;
  a.todo = c->view.todo;
  a.todo_count = c->view.todo_count + c->update_parity;
  a.todo_count_next = c->view.todo_count + (1 - c->update_parity);
  hipError_t e = qaq_launch_update(a, (a.len_after + QAQ_TT - 1) / QAQ_TT, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "qaq_decode_update");
  c->update_parity ^= 1;
  c->row_len[r.new_row] = a.len_after;
  c->ring_next = (r.new_row + 1) % c->dims.window;
  c->len = a.len_after;
  return QAQ_OK;
}

int qaq_prefill_window(qaq_cache* c, const void* dev_q_last, int32_t n_rows, const void* dev_k, int32_t T,
                       float* dev_scores_out, void* stream) {
  if (!c || !dev_q_last || !dev_k || !dev_scores_out) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  if (c->len != 0) return fail(QAQ_ERR_INVALID_ARG, "the cache already holds %d tokens", c->len);
  if (n_rows < 1 || n_rows > c->dims.window) return fail(QAQ_ERR_INVALID_ARG, "n_rows %d outside [1, window %d]", n_rows, c->dims.window);
  if (T - c->max_shortfall < n_rows) return fail(QAQ_ERR_INVALID_ARG, "prompt of %d tokens is shorter than %d rows", T - c->max_shortfall, n_rows);
  if (T > c->cfg.max_tokens) return fail(QAQ_ERR_CAPACITY, "prompt of %d tokens exceeds max_tokens %d", T, c->cfg.max_tokens);
  if (((uintptr_t)dev_q_last & 15) || ((uintptr_t)dev_k & 15)) return fail(QAQ_ERR_INVALID_ARG, "Q/K input must be 16-byte aligned");
  QaqPrefillArgs a;
  std::memset(&a, 0, sizeof(a));
  a.v = c->view;
  a.T = T;
  a.n_rows = n_rows;
  a.G = c->dims.Hq / c->dims.Hkv;
  a.q = (const __half*)dev_q_last;
  a.k = (const __half*)dev_k;
  a.scores = dev_scores_out;
  hipError_t e = qaq_launch_prefill_window(a, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "qaq_prefill_window");
  std::memset(c->row_len, 0, sizeof(c->row_len));
  for (int r = 0; r < n_rows; ++r) c->row_len[r] = T - n_rows + r + 1;
  c->ring_next = n_rows % c->dims.window;
  return QAQ_OK;
}

int qaq_quantize_append_selected(qaq_cache* c, const void* dev_k, const void* dev_v, int32_t n_new,
                                 uint8_t* dev_k_bits, uint8_t* dev_v_bits, void* stream) {
  if (!c) return fail(QAQ_ERR_INVALID_ARG, "cache is NULL");
  if (n_new < 0) return fail(QAQ_ERR_INVALID_ARG, "n_new is negative");
  if (n_new == 0) return QAQ_OK;
  if (!dev_k || !dev_v) return fail(QAQ_ERR_INVALID_ARG, "K/V input is NULL");
  if (((uintptr_t)dev_k & 15) || ((uintptr_t)dev_v & 15)) return fail(QAQ_ERR_INVALID_ARG, "K/V input must be 16-byte aligned");
  if ((long long)c->len + n_new > c->cfg.max_tokens)
    return fail(QAQ_ERR_CAPACITY, "%d cached + %d new tokens exceed max_tokens %d", c->len, n_new, c->cfg.max_tokens);
  if (first_append_too_short(c, n_new)) return QAQ_ERR_INVALID_ARG;
  QaqBuildArgs a;
  std::memset(&a, 0, sizeof(a));
  a.v = c->view;
  a.mode = 3;
  a.len_before = c->len;
  a.len_after = c->len + n_new;
  a.tile0 = first_open_tile(c);
  a.n_new = n_new;
  a.widest = c->cfg.bit_set[c->cfg.n_bits - 1];
  a.newx[0] = (const __half*)dev_k; a.newx[1] = (const __half*)dev_v;
  QaqRuleArgs& r = a.rule;
  r.G = c->dims.Hq / c->dims.Hkv;
  r.new_row = -1;
  for (int i = 0; i < QAQ_MAX_WINDOW; ++i) r.row_len[i] = i < c->dims.window ? c->row_len[i] : 0;
  r.nbits = c->cfg.n_bits;
  for (int i = 0; i < 5; ++i) r.bit_set[i] = c->cfg.bit_set[i < r.nbits ? i : r.nbits - 1];
  threshold_tables(c, a.len_after, r.tau_k, r.c_v);
  r.out_bits[0] = dev_k_bits; r.out_bits[1] = dev_v_bits;
  const int tile_last = (a.len_after - 1) / QAQ_TT;
  hipError_t e = qaq_launch_build(a, tile_last - a.tile0 + 1, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "qaq_quantize_append_selected");
  c->len = a.len_after;
  return QAQ_OK;
}

static int decode_attention(qaq_cache* c, const void* dev_q, const void* dev_k_new, const void* dev_v_new,
                            void* dev_out, int32_t out_is_fp32, float* dev_scores_out, void* stream, bool static_scratch) {
  if (!c || !dev_q || !dev_out) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  if ((dev_k_new == nullptr) != (dev_v_new == nullptr)) return fail(QAQ_ERR_INVALID_ARG, "k_new and v_new must be given together");
  if (c->len == 0 && !dev_k_new) return fail(QAQ_ERR_INVALID_ARG, "empty cache and no new token");
  QaqAttnArgs a;
  std::memset(&a, 0, sizeof(a));
  a.v = c->view;
  a.len = c->len;
  a.len_shortest = c->len > c->max_shortfall ? c->len - c->max_shortfall : 0;
  a.G = c->dims.Hq / c->dims.Hkv;
  a.q = (const __half*)dev_q;
  a.k_new = (const __half*)dev_k_new;
  a.v_new = (const __half*)dev_v_new;
  a.out = dev_out;
  a.out_is_fp32 = out_is_fp32;
  a.scores = dev_scores_out;
  a.score_stride = c->len + (dev_k_new ? 1 : 0);
  hipEvent_t* ev = nullptr;
  int kernels = 0;
  const bool timed = !c->prof_ev.empty() && (size_t)(4 * c->prof_n + 4) <= c->prof_ev.size();
  if (timed) ev = &c->prof_ev[4 * c->prof_n];
  bool too_big = false;
  hipError_t e = qaq_launch_attention(a, (hipStream_t)stream, ev, &kernels, static_scratch, &too_big);
  if (too_big)
    return fail(QAQ_ERR_CAPACITY, "qaq_decode_attention_static: the partial results of this shape (%d query heads x %d tiles) "
                "exceed the library's %zu-byte scratch array; use qaq_decode_attention", c->dims.B * c->dims.Hq,
                (c->len + QAQ_TT - 1) / QAQ_TT, qaq_static_scratch_bytes());
  if (timed && e == hipSuccess) c->prof_kernels[c->prof_n++] = kernels;
  if (e != hipSuccess) return hip_fail(e, "qaq_decode_attention");
  return QAQ_OK;
}

int qaq_decode_attention(qaq_cache* c, const void* dev_q, const void* dev_k_new, const void* dev_v_new,
                         void* dev_out, int32_t out_is_fp32, float* dev_scores_out, void* stream) {
  return decode_attention(c, dev_q, dev_k_new, dev_v_new, dev_out, out_is_fp32, dev_scores_out, stream, false);
}

int qaq_decode_attention_static(qaq_cache* c, const void* dev_q, const void* dev_k_new, const void* dev_v_new,
                                void* dev_out, int32_t out_is_fp32, float* dev_scores_out, void* stream) {
  return decode_attention(c, dev_q, dev_k_new, dev_v_new, dev_out, out_is_fp32, dev_scores_out, stream, true);
}

size_t qaq_static_scratch_limit(void) { return qaq_static_scratch_bytes(); }

int qaq_profile_begin(qaq_cache* c, int32_t max_calls) {
  if (!c || max_calls < 0 || max_calls > 4096) return fail(QAQ_ERR_INVALID_ARG, "bad profile request");
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  c->prof_ev.clear();
  c->prof_n = 0;
  c->prof_kernels.assign(max_calls, 0);
  for (int i = 0; i < 4 * max_calls; ++i) {
    hipEvent_t e;
    hipError_t r = hipEventCreate(&e);
    if (r != hipSuccess) return hip_fail(r, "qaq_profile_begin");
    c->prof_ev.push_back(e);
  }
  return QAQ_OK;
}

int qaq_profile_read(qaq_cache* c, float* host_ms_tile, float* host_ms_merge, int32_t* n_calls) {
  if (!c || !host_ms_tile || !host_ms_merge || !n_calls) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  *n_calls = c->prof_n;
  for (int i = 0; i < c->prof_n; ++i) {
    const int k = c->prof_kernels[i];
    host_ms_tile[i] = host_ms_merge[i] = 0.0f;
    hipError_t r = hipSuccess;
    if (k >= 1) r = hipEventSynchronize(c->prof_ev[4 * i + (k == 2 ? 3 : 1)]);
    if (k >= 1 && r == hipSuccess) r = hipEventElapsedTime(&host_ms_tile[i], c->prof_ev[4 * i], c->prof_ev[4 * i + 1]);
    if (k == 2 && r == hipSuccess) r = hipEventElapsedTime(&host_ms_merge[i], c->prof_ev[4 * i + 1], c->prof_ev[4 * i + 3]);
    if (r != hipSuccess) return hip_fail(r, "qaq_profile_read");
  }
  c->prof_n = 0;
  return QAQ_OK;
}

int qaq_dequantize(qaq_cache* c, int32_t t0, int32_t t1, void* dev_k_out, void* dev_v_out, void* stream) {
  if (!c) return fail(QAQ_ERR_INVALID_ARG, "cache is NULL");
  if (t0 < 0 || t1 < t0 || t1 > c->len) return fail(QAQ_ERR_INVALID_ARG, "bad range [%d, %d) for %d tokens", t0, t1, c->len);
  if (t1 == t0 || (!dev_k_out && !dev_v_out)) return QAQ_OK;
  QaqDequantArgs a;
  std::memset(&a, 0, sizeof(a));
  a.v = c->view;
  a.len = c->len; a.t0 = t0; a.t1 = t1;
  a.out[0] = (__half*)dev_k_out; a.out[1] = (__half*)dev_v_out;
  hipError_t e = qaq_launch_dequant(a, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "qaq_dequantize");
  return QAQ_OK;
}

int qaq_export_canonical(qaq_cache* c, int32_t side, uint8_t* dev_bits, void* dev_minmax, uint8_t* dev_oidx,
                         void* dev_oval, uint8_t* dev_codes, void* stream) {
  if (!c) return fail(QAQ_ERR_INVALID_ARG, "cache is NULL");
  if (side != 0 && side != 1) return fail(QAQ_ERR_INVALID_ARG, "side must be 0 (keys) or 1 (values)");
  if (c->len == 0) return QAQ_OK;
  QaqExportArgs a;
  std::memset(&a, 0, sizeof(a));
  a.v = c->view;
  a.len = c->len; a.side = side;
  a.bits = dev_bits; a.minmax = (uint16_t*)dev_minmax; a.oidx = dev_oidx; a.oval = (uint16_t*)dev_oval; a.codes = dev_codes;
  hipError_t e = qaq_launch_export(a, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "qaq_export_canonical");
  return QAQ_OK;
}

int qaq_stats(qaq_cache* c, qaq_stats_t* out, void* stream) {
  if (!c || !out) return fail(QAQ_ERR_INVALID_ARG, "NULL argument");
  std::memset(out, 0, sizeof(*out));
  out->tokens = c->len;
  long long buf[16] = {0};
  uint32_t handed[2] = {0, 0};
  hipError_t e = qaq_launch_stats(c->view, c->len, (hipStream_t)stream);
  if (e == hipSuccess) e = hipMemcpyAsync(handed, c->view.todo_count, sizeof(handed), hipMemcpyDeviceToHost, (hipStream_t)stream);
  if (e == hipSuccess) e = hipMemcpyAsync(buf, c->view.statbuf, sizeof(buf), hipMemcpyDeviceToHost, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "qaq_stats");
  static const int widths[4] = {2, 3, 4, 8};
  const long long D = c->dims.D;
  for (int i = 0; i < 4; ++i) {
    out->hist_k[i] = buf[i];
    out->hist_v[i] = buf[4 + i];
    out->code_bytes += (buf[i] + buf[4 + i]) * D * widths[i] / 8;
  }
  out->hist_k[4] = buf[10];
  out->hist_v[4] = buf[11];
  out->code_bytes += (buf[10] + buf[11]) * D / 8;
  out->layout_code_bytes = buf[8];
  out->meta_bytes = buf[9];
  long long seq_tokens = 0;
  for (int b = 0; b < c->dims.B; ++b) seq_tokens += seq_len(c, b, c->len);
  out->fp16_bytes = seq_tokens * c->dims.Hkv * D * 2 * 2;
  out->update_handovers = (long long)handed[0] + handed[1];     // (the counter of the step to come is zero)
  out->refused_upgrades = buf[12];
  out->served_upgrades = buf[13];
  return QAQ_OK;
}

int qaq_host_alloc(size_t bytes, void** host_ptr, void** dev_ptr) {
  if (!host_ptr || !dev_ptr || bytes == 0) return fail(QAQ_ERR_INVALID_ARG, "qaq_host_alloc: NULL argument or zero size");
  *host_ptr = *dev_ptr = nullptr;
  void* h = nullptr;
  hipError_t e = hipHostMalloc(&h, bytes, hipHostMallocMapped | hipHostMallocPortable);
  if (e != hipSuccess) return hip_fail(e, "qaq_host_alloc");
  void* d = nullptr;
  e = hipHostGetDevicePointer(&d, h, 0);
  if (e != hipSuccess) { (void)hipHostFree(h); return hip_fail(e, "qaq_host_alloc: device address"); }
  *host_ptr = h;
  *dev_ptr = d;
  return QAQ_OK;
}

int qaq_host_free(void* host_ptr) {
  if (!host_ptr) return QAQ_OK;
  hipError_t e = hipHostFree(host_ptr);
  if (e != hipSuccess) return hip_fail(e, "qaq_host_free");
  return QAQ_OK;
}

int qaq_stream_read(const void* dev_src, size_t bytes, uint32_t* dev_sink, void* stream) {
  if (!dev_src || !dev_sink || (bytes & 15) || ((uintptr_t)dev_src & 15)) return fail(QAQ_ERR_INVALID_ARG, "qaq_stream_read: NULL or unaligned argument");
  if (bytes == 0) return QAQ_OK;
  hipLaunchKernelGGL(k_stream_read, dim3(4096), dim3(256), 0, (hipStream_t)stream, (const u32x4*)dev_src, bytes / 16, dev_sink);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? QAQ_OK : hip_fail(e, "qaq_stream_read");
}

int qaq_stream_copy(void* dev_dst, const void* dev_src, size_t bytes, void* stream) {
  if (!dev_src || !dev_dst || (bytes & 15) || ((uintptr_t)dev_src & 15) || ((uintptr_t)dev_dst & 15))
    return fail(QAQ_ERR_INVALID_ARG, "qaq_stream_copy: NULL or unaligned argument");
  if (bytes == 0) return QAQ_OK;
  hipLaunchKernelGGL(k_stream_copy, dim3(2048), dim3(256), 0, (hipStream_t)stream, (u32x4*)dev_dst, (const u32x4*)dev_src, bytes / 16);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? QAQ_OK : hip_fail(e, "qaq_stream_copy");
}

// Host-only view of the code layout, for layout tests: where the field of width
// `bf` (1, 2, 4 or 8) of token `idx` of its region, channel d, is stored, relative to the
// start of the tile side; the region offsets follow from the class counts.
int qaq_debug_field(int32_t side, int32_t D, int32_t n3, int32_t n2, int32_t n4, int32_t n8, int32_t n1, int32_t bf,
                    int32_t idx, int32_t d, uint32_t* byte_off, int32_t* shift, uint32_t* region_end) {
  if ((D != 64 && D != 128) || d < 0 || d >= D || idx < 0) return fail(QAQ_ERR_INVALID_ARG, "bad layout query");
  QaqCounts c; c.n3 = n3; c.n2 = n2; c.n4 = n4; c.n8 = n8; c.n1 = n1;
  QaqFieldPos p;
  const int fw = bf == 0 ? 1 : bf;      // field width; bf 0 = the region of the 1-bit tokens
  if (side == 0) {
    const QaqKRegions r = qaq_k_regions(c, D);
    const uint32_t ro = bf == 2 ? r.r2 : bf == 1 ? r.r1 : bf == 4 ? r.r4 : bf == 8 ? r.r8 : r.r1b;
    p = qaq_k_field(ro, fw, idx, d, D);
    *region_end = r.end;
  } else {
    const QaqVRegions r = qaq_v_regions(c, D);
    if (bf == 8) { p.byte_off = (r.r8 + (uint32_t)idx * D + d) & ~3u; p.shift = 8 * (d & 3); }
    else p = qaq_v_field(bf == 2 ? r.r2 : bf == 1 ? r.r1 : bf == 4 ? r.r4 : r.r1b, fw, idx, d, D);
    *region_end = r.end;
  }
  *byte_off = p.byte_off;
  *shift = p.shift;
  return QAQ_OK;
}

uint32_t qaq_debug_tile_capacity(int32_t side, int32_t D) { return side == 0 ? qaq_k_cap(D) : qaq_v_cap(D); }

}  // extern "C"
