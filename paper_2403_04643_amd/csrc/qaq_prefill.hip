// Prompt encoding: the last n causal score rows of a prompt, from the unquantized fp16
// keys, installed as the attention window (Section 2.1 prompt encoding; Section 4.2
// "attention window").
//
// Per KV head this is a dense contraction [G*n query rows x D] . [D x T keys], so it runs on
// the fp16 matrix instruction (fp32 accumulation; products of fp16 numbers are exact in
// fp32).  k_prefill_logits reads every key once: a wavefront keeps 64 keys in registers as B
// operands and sweeps the query rows of the head over them in blocks of 16.  It leaves
// logit/sqrt(D) (minus infinity where a token lies after the query's position) in the score
// buffer; k_prefill_softmax turns each row into scores in place and writes the maximum over
// the query heads of a KV head into the ring rows.
#include "qaq_internal.h"

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;
constexpr int kKeep = 16;          // logits per thread the softmax kernel keeps in registers (a 4096-token row)

// tokens a query row attends to: row i belongs to position T - n + i of a prompt of T tokens
__device__ __forceinline__ int row_length(int T, int n, int i) { return T - n + i + 1; }

template <int D>
__global__ __launch_bounds__(kThreads) void k_prefill_logits(QaqPrefillArgs a) {
  constexpr int NS = D / 32;       // matrix instructions along the head dimension
  const QaqView& v = a.v;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, kb = lane >> 4;
  const int bh = blockIdx.x, b = bh / v.Hkv, h = bh % v.Hkv;     // heads fastest (see k_build)
  const int t_wave = blockIdx.y * QAQ_TT + 64 * wave;
  if (t_wave >= a.T) return;
  const int T_seq = qaq_seq_len(v, b, a.T);      // tokens of this sequence's prompt (rows of K past them are padding)

  // 64 keys of this wavefront: lane (col, kb) holds channels 32s + 8kb .. +8 of key 16g + col
  h8 key[4][NS];
  const __half* kbase = a.k + (size_t)bh * a.T * D;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int t = min(t_wave + 16 * g + col, a.T - 1);    // clamped: the tail reads a valid row and is masked below
#pragma unroll
    for (int s = 0; s < NS; ++s) key[g][s] = __builtin_nontemporal_load((const h8*)(kbase + (size_t)t * D + 32 * s + 8 * kb));
  }

  const int R = a.G * a.n_rows;    // query rows of this KV head: (query head g, prompt row i) -> g * n + i
  const float scale = rsqrtf((float)D);
  for (int r0 = 0; r0 < R; r0 += 16) {
    h8 qa[NS];
    {
      const int r = r0 + col;
      const bool live = r < R;
      const int hq = h * a.G + (live ? r / a.n_rows : 0), i = live ? r % a.n_rows : 0;
      const __half* qrow = a.q + (((size_t)b * v.Hq + hq) * a.n_rows + i) * D;
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        qa[s] = *(const h8*)(qrow + 32 * s + 8 * kb);
        if (!live) qa[s] = (h8)(_Float16)0;
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      f4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int s = 0; s < NS; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[s], key[g][s], acc, 0, 0, 0);
      const int t = t_wave + 16 * g + col;
      if (t < a.T) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {      // element j of the result: query row 4kb + j of the block, key `col`
          const int r = r0 + 4 * kb + j;
          if (r < R) {
            const int hq = h * a.G + r / a.n_rows, i = r % a.n_rows;
            a.scores[(((size_t)i * v.B + b) * v.Hq + hq) * a.T + t] =
                t < row_length(T_seq, a.n_rows, i) ? acc[j] * scale : -INFINITY;
          }
        }
      }
    }
  }
}

__device__ __forceinline__ float block_reduce(float x, bool is_max, float* red) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float y = __shfl_xor(x, o);
    x = is_max ? fmaxf(x, y) : x + y;
  }
  __syncthreads();                 // red[] may still be read from the previous reduction
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return is_max ? fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) : (red[0] + red[1]) + (red[2] + red[3]);
}

// One workgroup per (prompt row, sequence, KV head): softmax of each of its G query heads'
// logit rows in place, and the ring row = maximum over the G heads.
__global__ __launch_bounds__(kThreads) void k_prefill_softmax(QaqPrefillArgs a) {
  __shared__ float red[4];
  const QaqView& v = a.v;
  const int tid = threadIdx.x;
  const int i = blockIdx.x, bh = blockIdx.y, b = bh / v.Hkv, h = bh % v.Hkv;
  const int len = row_length(qaq_seq_len(v, b, a.T), a.n_rows, i);
  const size_t ring_row = (size_t)v.B * v.Hkv * v.Tmax;
  const size_t ring0 = (size_t)i * ring_row + qaq_bh(v, b, h) * v.Tmax;
  for (int g = 0; g < a.G; ++g) {
    float* row = a.scores + (((size_t)i * v.B + b) * v.Hq + (h * a.G + g)) * a.T;
    // maximum and sum in one sweep: every thread keeps its logits (T / 256 of them, at most
    // kKeep in registers, the rest is read again), its own maximum and the sum against it
    float mine[kKeep];
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
      const int t = tid + k * kThreads;
      mine[k] = t < len ? row[t] : -INFINITY;
      m = fmaxf(m, mine[k]);
    }
    for (int t = tid + kKeep * kThreads; t < len; t += kThreads) m = fmaxf(m, row[t]);
    m = block_reduce(m, true, red);
    float l = 0.0f;
#pragma unroll
    for (int k = 0; k < kKeep; ++k) l += expf(mine[k] - m);        // exp(-inf) = 0 past the row's end
    for (int t = tid + kKeep * kThreads; t < len; t += kThreads) l += expf(row[t] - m);
    l = block_reduce(l, false, red);
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
      const int t = tid + k * kThreads;
      if (t < a.T) {
        const float s = t < len ? expf(mine[k] - m) / l : 0.0f;
        row[t] = s;
        if (t < len) qaq_ring_store(v, ring0 + t, g == 0 ? s : fmaxf(qaq_ring_load(v, ring0 + t), s));   // thread tid is the only one to touch position t
      }
    }
    for (int t = tid + kKeep * kThreads; t < a.T; t += kThreads) {
      const float s = t < len ? expf(row[t] - m) / l : 0.0f;
      row[t] = s;
      if (t < len) qaq_ring_store(v, ring0 + t, g == 0 ? s : fmaxf(qaq_ring_load(v, ring0 + t), s));
    }
  }
}

}  // namespace

hipError_t qaq_launch_prefill_window(const QaqPrefillArgs& a, hipStream_t s) {
  const QaqView& v = a.v;
  const dim3 grid(v.B * v.Hkv, (a.T + QAQ_TT - 1) / QAQ_TT);
  if (v.D == 128) hipLaunchKernelGGL(k_prefill_logits<128>, grid, dim3(kThreads), 0, s, a);
  else if (v.D == 64) hipLaunchKernelGGL(k_prefill_logits<64>, grid, dim3(kThreads), 0, s, a);
  else return hipErrorInvalidValue;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_prefill_softmax, dim3(a.n_rows, v.B * v.Hkv), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}
