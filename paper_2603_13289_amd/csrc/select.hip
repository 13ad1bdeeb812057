// K5: token selection from the deviation scores.  One workgroup per request.
//   * budget selection: the k largest scores, equal scores to the lower index, ascending output
//   * threshold selection (Eq. 5 / Eq. 7): score >= tau * mean(score)
#include "common.h"

namespace rc {

static constexpr int kSelThreads = 1024;
static constexpr int kSelWaves = kSelThreads / 64;

// Monotone map float -> uint32 (larger float => larger key).  -0 and +0 map to the same key so that
// they tie; NaNs with the sign bit clear order above +inf.
__device__ inline uint32_t order_key(float f) {
  if (f == 0.0f) f = 0.0f;
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive prefix sum of one int per thread over the block; also returns the block total
__device__ inline int block_exclusive_scan(int v, int* lds /* kSelWaves + 1 ints */, int* total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) lds[w] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < kSelWaves; ++i) {
      const int t = lds[i];
      lds[i] = run;
      run += t;
    }
    lds[kSelWaves] = run;
  }
  __syncthreads();
  *total = lds[kSelWaves];
  return lds[w] + inc - v;
}

__device__ __forceinline__ void topk_body(const float* __restrict__ score, int n, int k, int* __restrict__ idx_out) {
  __shared__ int hist[256];
  __shared__ int scan_lds[kSelWaves + 1];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;
  if (k <= 0) return;

  // radix select, 8 bits at a time from the top: find the key of the k-th largest element
  uint32_t prefix = 0, mask = 0;
  int need = k;  // rank (1-based, from the top) still to be located inside the current prefix class
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = threadIdx.x; i < 256; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += kSelThreads) {
      const uint32_t key = order_key(score[i]);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int run = 0, d = 255;
      for (; d > 0; --d) {
        if (run + hist[d] >= need) break;
        run += hist[d];
      }
      s_prefix = prefix | ((uint32_t)d << shift);
      s_need = need - run;
    }
    __syncthreads();
    prefix = s_prefix;
    need = s_need;
    mask |= 255u << shift;
    __syncthreads();
  }
  // prefix is now the threshold key; `need` of the elements equal to it are taken, lowest indices first

  // ordered compaction: each thread owns a contiguous run of indices
  const int chunk = (n + kSelThreads - 1) / kSelThreads;
  const int lo = min(threadIdx.x * chunk, n), hi = min(lo + chunk, n);
  int n_gt = 0, n_eq = 0;
  for (int i = lo; i < hi; ++i) {
    const uint32_t key = order_key(score[i]);
    n_gt += key > prefix;
    n_eq += key == prefix;
  }
  int total;
  const int eq_before = block_exclusive_scan(n_eq, scan_lds, &total);
  const int eq_take = min(max(need - eq_before, 0), n_eq);
  int out = block_exclusive_scan(n_gt + eq_take, scan_lds, &total);
  int eq_left = eq_take;
  for (int i = lo; i < hi; ++i) {
    const uint32_t key = order_key(score[i]);
    if (key > prefix) {
      idx_out[out++] = i;
    } else if (key == prefix && eq_left > 0) {
      idx_out[out++] = i;
      --eq_left;
    }
  }
}

__global__ void __launch_bounds__(kSelThreads)
topk_kernel(const float* __restrict__ score, int n, int k, int* __restrict__ idx_out) {
  topk_body(score, n, k, idx_out);
}

// one workgroup per request of a call; requests without a budget (or not in the dense phase) are skipped
__global__ void __launch_bounds__(kSelThreads)
topk_batch_kernel(const float* __restrict__ scores, const ReqTable* __restrict__ table, int* __restrict__ sel_idx) {
  const ReqDev& rq = table->r[blockIdx.x];
  if (rq.k <= 0 || rq.S <= 0) return;      // uniform for the workgroup
  topk_body(scores + rq.score_base, rq.S, min(rq.k, rq.S), sel_idx + rq.sel_base);
}

hipError_t launch_topk_batch(const float* scores, const ReqTable* table, int n_req, int* sel_idx, hipStream_t st) {
  if (n_req <= 0) return hipSuccess;
  topk_batch_kernel<<<n_req, kSelThreads, 0, st>>>(scores, table, sel_idx);
  return hipGetLastError();
}

__global__ void __launch_bounds__(256)
copy_sel_batch_kernel(const int* __restrict__ forced, const ReqTable* __restrict__ table, int* __restrict__ sel_idx) {
  const ReqDev& rq = table->r[blockIdx.y];
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rq.k) sel_idx[rq.sel_base + i] = forced[rq.sel_base + i];
}

hipError_t launch_copy_sel_batch(const int* forced, const ReqTable* table, int n_req, int* sel_idx, hipStream_t st) {
  if (n_req <= 0) return hipSuccess;
  // k <= S <= 2^20 entries per request
  copy_sel_batch_kernel<<<dim3(4096, (unsigned)n_req), 256, 0, st>>>(forced, table, sel_idx);
  return hipGetLastError();
}

hipError_t launch_topk(const float* score, int n, int k, int* idx_out, hipStream_t st) {
  if (k <= 0 || n <= 0) return hipSuccess;
  topk_kernel<<<1, kSelThreads, 0, st>>>(score, n, k, idx_out);
  return hipGetLastError();
}

// Eq. (5)/(7).  The mean is accumulated in double in a fixed order, so the comparison
// score >= tau * mean is decided in double on exactly representable inputs.
__global__ void __launch_bounds__(kSelThreads)
threshold_select_kernel(const float* __restrict__ score, int n, float tau, int* __restrict__ idx_out,
                        int* __restrict__ count_out) {
  __shared__ double part[kSelWaves];
  __shared__ int scan_lds[kSelWaves + 1];
  __shared__ double s_thr;
  double acc = 0.0;
  for (int i = threadIdx.x; i < n; i += kSelThreads) acc += (double)score[i];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int i = 0; i < kSelWaves; ++i) s += part[i];
    s_thr = (double)tau * (s / (double)n);
  }
  __syncthreads();
  const double thr = s_thr;
  const int chunk = (n + kSelThreads - 1) / kSelThreads;
  const int lo = min(threadIdx.x * chunk, n), hi = min(lo + chunk, n);
  int cnt = 0;
  for (int i = lo; i < hi; ++i) cnt += (double)score[i] >= thr;
  int total;
  int out = block_exclusive_scan(cnt, scan_lds, &total);
  for (int i = lo; i < hi; ++i)
    if ((double)score[i] >= thr) idx_out[out++] = i;
  if (threadIdx.x == 0) *count_out = total;
}

// Eq. (5)-(10) in one pass: I_dev (deviation >= tau_dev * mean) united with I_inf-score (influence >=
// tau_inf * mean, when influence scores are given) and the last k_suf tokens; ascending; count out.
// Means are accumulated in double in a fixed order, comparisons are made in double.
__device__ __forceinline__ void final_select_body(const float* __restrict__ s_dev, const float* __restrict__ s_inf, int n,
                                                  float tau_dev, float tau_inf, int k_suf, int* __restrict__ idx_out,
                                                  int* __restrict__ count_out) {
  __shared__ double part[2][kSelWaves];
  __shared__ int scan_lds[kSelWaves + 1];
  __shared__ double s_thr[2];
  double a = 0.0, b = 0.0;
  for (int i = threadIdx.x; i < n; i += kSelThreads) {
    a += (double)s_dev[i];
    if (s_inf) b += (double)s_inf[i];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    a += __shfl_xor(a, o, 64);
    b += __shfl_xor(b, o, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    part[0][threadIdx.x >> 6] = a;
    part[1][threadIdx.x >> 6] = b;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double sa = 0.0, sb = 0.0;
    for (int i = 0; i < kSelWaves; ++i) { sa += part[0][i]; sb += part[1][i]; }
    s_thr[0] = (double)tau_dev * (sa / (double)n);
    s_thr[1] = (double)tau_inf * (sb / (double)n);
  }
  __syncthreads();
  const double thr_dev = s_thr[0], thr_inf = s_thr[1];
  const int chunk = (n + kSelThreads - 1) / kSelThreads;
  const int lo = min(threadIdx.x * chunk, n), hi = min(lo + chunk, n);
  auto chosen = [&](int i) {
    return (double)s_dev[i] >= thr_dev || (s_inf && (double)s_inf[i] >= thr_inf) || i >= n - k_suf;
  };
  int cnt = 0;
  for (int i = lo; i < hi; ++i) cnt += chosen(i);
  int total;
  int out = block_exclusive_scan(cnt, scan_lds, &total);
  for (int i = lo; i < hi; ++i)
    if (chosen(i)) idx_out[out++] = i;
  if (threadIdx.x == 0) *count_out = total;
}

__global__ void __launch_bounds__(kSelThreads)
final_select_kernel(const float* __restrict__ s_dev, const float* __restrict__ s_inf, int n, float tau_dev,
                    float tau_inf, int k_suf, int* __restrict__ idx_out, int* __restrict__ count_out) {
  final_select_body(s_dev, s_inf, n, tau_dev, tau_inf, k_suf, idx_out, count_out);
}

__global__ void __launch_bounds__(kSelThreads)
final_select_batch_kernel(const float* __restrict__ scores, InfluenceIn inf, const ReqTable* __restrict__ table,
                          float tau_dev, float tau_inf, int k_suf, int* __restrict__ sel_idx,
                          int* __restrict__ sel_cnt) {
  const ReqDev& rq = table->r[blockIdx.x];
  if (rq.k <= 0 || rq.S <= 0) return;
  final_select_body(scores + rq.score_base, inf.s_inf[blockIdx.x], rq.S, tau_dev, tau_inf, k_suf,
                    sel_idx + rq.sel_base, sel_cnt + blockIdx.x);
}

hipError_t launch_final_select_batch(const float* scores, const InfluenceIn& inf, const ReqTable* table, int n_req,
                                     float tau_dev, float tau_inf, int k_suf, int* sel_idx, int* sel_cnt,
                                     hipStream_t st) {
  if (n_req <= 0) return hipSuccess;
  final_select_batch_kernel<<<n_req, kSelThreads, 0, st>>>(scores, inf, table, tau_dev, tau_inf, k_suf, sel_idx, sel_cnt);
  return hipGetLastError();
}

hipError_t launch_final_select(const float* s_dev, const float* s_inf, int n, float tau_dev, float tau_inf, int k_suf,
                               int* idx_out, int* count_out, hipStream_t st) {
  final_select_kernel<<<1, kSelThreads, 0, st>>>(s_dev, s_inf, n, tau_dev, tau_inf, k_suf, idx_out, count_out);
  return hipGetLastError();
}

hipError_t launch_threshold_select(const float* score, int n, float tau, int* idx_out, int* count_out,
                                   hipStream_t st) {
  threshold_select_kernel<<<1, kSelThreads, 0, st>>>(score, n, tau, idx_out, count_out);
  return hipGetLastError();
}

}  // namespace rc
