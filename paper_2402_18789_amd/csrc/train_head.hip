// The two ends of a finetuning step around the decoder layers: the generative loss of a forward
// window (Alg. 2, forward loop: final norm, LM head, next-token cross-entropy) with the gradient
// the backward pass starts from, and the Adam update of the bypass-network parameters (the
// optimizer the paper's setup names).
//
//   loss head:  h = rmsnorm(x; g)                      (norm kernel of the layer)
//               z = h W_lm^T            [n, V]         (forward-form GEMM of the layer)
//               row i: lse_i = logsumexp(z_i); loss_i = lse_i - z_i[y_i];
//                      z_i <- scale (softmax(z_i) - onehot(y_i))      in place, one block per row
//               dh = dz W_lm            [n, H]         (input-gradient GEMM, K = V split across blocks)
//               dx = rmsnorm_bwd(x; g, dh)
//   Row losses are summed by one block in a fixed order and added to the caller's accumulator:
//   the result does not depend on scheduling.
#include "flexco_internal.h"
#include "device_types.h"

namespace flexco {

namespace {

constexpr int CE_THREADS = 512;

__device__ inline void combine(float& m, float& s, float m2, float s2) {
  const float mx = fmaxf(m, m2);
  if (mx == -INFINITY) return;                    // both empty
  s = s * __expf(m - mx) + s2 * __expf(m2 - mx);
  m = mx;
}

// one block per row: online (max, sum) pass, then the in-place gradient pass
template <typename T, bool VEC>
__global__ __launch_bounds__(CE_THREADS) void ce_rows_kernel(T* __restrict__ z, const int32_t* __restrict__ targets,
                                                             float* __restrict__ row_loss, int V, float scale) {
  constexpr int N = VEC ? Vec<T>::N : 1;
  __shared__ float red_m[CE_THREADS / 64], red_s[CE_THREADS / 64];
  __shared__ float lse_sh;
  T* zr = z + (size_t)blockIdx.x * V;
  int y = targets[blockIdx.x];
  if (y >= V) y = -1;                             // a target outside the vocabulary is treated as "no target"
  float m = -INFINITY, s = 0.f;
  for (int i = threadIdx.x * N; i < V; i += CE_THREADS * N) {
    float v[N];
    if (VEC) Vec<T>::load(zr + i, v); else v[0] = ld(zr + i);
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const float mx = fmaxf(m, v[j]);
      s = s * __expf(m - mx) + __expf(v[j] - mx);
      m = mx;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) combine(m, s, __shfl_xor(m, o, 64), __shfl_xor(s, o, 64));
  if ((threadIdx.x & 63) == 0) { red_m[threadIdx.x >> 6] = m; red_s[threadIdx.x >> 6] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float mm = red_m[0], ss = red_s[0];
    for (int w = 1; w < CE_THREADS / 64; ++w) combine(mm, ss, red_m[w], red_s[w]);
    const float lse = mm + __logf(ss);
    lse_sh = lse;
    row_loss[blockIdx.x] = y >= 0 ? lse - ld(zr + y) : 0.f;
  }
  __syncthreads();
  const float lse = lse_sh;
  const float sc = y >= 0 ? scale : 0.f;          // rows without a target contribute nothing
  for (int i = threadIdx.x * N; i < V; i += CE_THREADS * N) {
    float v[N];
    if (VEC) Vec<T>::load(zr + i, v); else v[0] = ld(zr + i);
#pragma unroll
    for (int j = 0; j < N; ++j) v[j] = sc * (__expf(v[j] - lse) - (i + j == y ? 1.f : 0.f));
    if (VEC) Vec<T>::store(zr + i, v); else st(zr + i, v[0]);
  }
}

// *accum += scale * sum_i row_loss[i], rows added in index order by strided partial sums of one block
__global__ __launch_bounds__(256) void loss_sum_kernel(const float* __restrict__ row_loss, int n, float scale,
                                                       float* __restrict__ accum) {
  __shared__ float part[256];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += row_loss[i];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) accum[0] += scale * part[0];
}

template <typename T>
__global__ __launch_bounds__(256) void adam_kernel(T* __restrict__ param, float* __restrict__ master,
                                                   const float* __restrict__ grad, float* __restrict__ m,
                                                   float* __restrict__ v, size_t n, float lr, float b1, float b2,
                                                   float eps, float corr1, float corr2) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float g = grad[i];
  const float mi = b1 * m[i] + (1.f - b1) * g;
  const float vi = b2 * v[i] + (1.f - b2) * g * g;
  m[i] = mi;
  v[i] = vi;
  float p = master ? master[i] : ld(param + i);
  p -= lr * (mi / corr1) / (sqrtf(vi / corr2) + eps);
  if (master) master[i] = p;
  st(param + i, p);
}

struct HeadWs {
  void *h, *z, *dh;
  float *row_loss, *part;
  size_t part_elems, bytes;
};

HeadWs carve_head(const flexco_lm_head& hd, int n, void* base) {
  const size_t e = esize(hd.dtype);
  char* p = (char*)base;
  size_t off = 0;
  auto take = [&](size_t bytes) { void* q = base ? p + off : nullptr; off += align_up(bytes, 256); return q; };
  HeadWs w;
  w.h = take(e * (size_t)n * hd.hidden);
  w.z = take(e * (size_t)n * hd.vocab);
  w.dh = take(e * (size_t)n * hd.hidden);
  w.row_loss = (float*)take(sizeof(float) * (size_t)n);
  w.part_elems = hd.dtype == FLEXCO_BF16 ? (size_t)16 * n * hd.hidden : 0;
  w.part = (float*)take(sizeof(float) * w.part_elems);
  w.bytes = off;
  return w;
}

int32_t check_head(const flexco_lm_head* hd) {
  FLEXCO_CHECK(hd, FLEXCO_EINVAL, "NULL head");
  FLEXCO_CHECK(hd->hidden > 0 && hd->vocab > 0, FLEXCO_EINVAL, "hidden and vocab must be positive");
  FLEXCO_CHECK(hd->dtype == FLEXCO_F32 || hd->dtype == FLEXCO_BF16, FLEXCO_EINVAL, "unknown dtype %d", hd->dtype);
  FLEXCO_CHECK(hd->g_final && hd->w_lm, FLEXCO_EINVAL, "NULL weight");
  FLEXCO_CHECK(aligned16(hd->g_final) && aligned16(hd->w_lm), FLEXCO_EINVAL, "misaligned weight");
  return FLEXCO_OK;
}

int32_t post(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FLEXCO_EHIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return FLEXCO_OK;
}

}  // namespace

}  // namespace flexco

using namespace flexco;

extern "C" int32_t flexco_lm_loss_workspace_bytes(const flexco_lm_head* head, int32_t n_max, size_t* out_bytes) {
  clear_error();
  FLEXCO_TRY(check_head(head));
  FLEXCO_CHECK(n_max >= 0 && out_bytes, FLEXCO_EINVAL, "bad argument");
  *out_bytes = carve_head(*head, n_max, nullptr).bytes;
  return FLEXCO_OK;
}

extern "C" int32_t flexco_lm_loss(const flexco_lm_head* head, const void* x, const int32_t* targets, int32_t n,
                                  float scale, float* loss_accum, void* dX, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  FLEXCO_TRY(check_head(head));
  FLEXCO_CHECK(n >= 0, FLEXCO_EINVAL, "n must be non-negative");
  if (n == 0) return FLEXCO_OK;
  FLEXCO_CHECK(x && targets && loss_accum && dX && ws, FLEXCO_EINVAL, "NULL argument");
  FLEXCO_CHECK(aligned16(x) && aligned16(dX) && aligned16(ws), FLEXCO_EINVAL, "misaligned pointer");
  const flexco_lm_head& hd = *head;
  HeadWs k = carve_head(hd, n, ws);
  FLEXCO_CHECK(k.bytes <= ws_bytes, FLEXCO_EWORKSPACE, "loss head needs %zu workspace bytes, got %zu", k.bytes, ws_bytes);
  hipStream_t s = (hipStream_t)stream;
  const int H = hd.hidden, V = hd.vocab, dt = hd.dtype;
  FLEXCO_TRY(launch_rmsnorm(x, hd.g_final, k.h, n, H, hd.rms_eps, dt, s));
  FLEXCO_TRY(launch_gemm(k.h, hd.w_lm, k.z, nullptr, nullptr, n, V, H, H, H, V, 0, false, dt, s, nullptr, nullptr, 0));
  {
    KernelTimerScope ts(FLEXCO_K_ELEMWISE, s);
    const bool vec = V % (dt == FLEXCO_BF16 ? 8 : 4) == 0;   // rows of z then start 16-byte aligned
    if (dt == FLEXCO_BF16) {
      if (vec) hipLaunchKernelGGL((ce_rows_kernel<bf16_t, true>), dim3(n), dim3(CE_THREADS), 0, s, (bf16_t*)k.z, targets, k.row_loss, V, scale);
      else hipLaunchKernelGGL((ce_rows_kernel<bf16_t, false>), dim3(n), dim3(CE_THREADS), 0, s, (bf16_t*)k.z, targets, k.row_loss, V, scale);
    } else {
      if (vec) hipLaunchKernelGGL((ce_rows_kernel<float, true>), dim3(n), dim3(CE_THREADS), 0, s, (float*)k.z, targets, k.row_loss, V, scale);
      else hipLaunchKernelGGL((ce_rows_kernel<float, false>), dim3(n), dim3(CE_THREADS), 0, s, (float*)k.z, targets, k.row_loss, V, scale);
    }
    FLEXCO_TRY(post("ce_rows"));
    hipLaunchKernelGGL(loss_sum_kernel, dim3(1), dim3(256), 0, s, k.row_loss, n, scale, loss_accum);
    FLEXCO_TRY(post("loss_sum"));
  }
  FLEXCO_TRY(launch_gemm(k.z, hd.w_lm, k.dh, nullptr, nullptr, n, H, V, V, H, H, 0, true, dt, s, nullptr, k.part, k.part_elems));
  FLEXCO_TRY(launch_rmsnorm_bwd(x, hd.g_final, k.dh, nullptr, dX, n, H, hd.rms_eps, dt, s));
  return FLEXCO_OK;
}

extern "C" int32_t flexco_adam_step(void* param, float* master, const float* grad, float* m, float* v, size_t n,
                                    int32_t dtype, float lr, float beta1, float beta2, float eps, int32_t step,
                                    void* stream) {
  clear_error();
  FLEXCO_CHECK(dtype == FLEXCO_F32 || dtype == FLEXCO_BF16, FLEXCO_EINVAL, "unknown dtype %d", dtype);
  FLEXCO_CHECK(step >= 1, FLEXCO_EINVAL, "step counts from 1 (got %d)", step);
  FLEXCO_CHECK(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f, FLEXCO_EINVAL, "beta outside [0, 1)");
  if (n == 0) return FLEXCO_OK;
  FLEXCO_CHECK(param && grad && m && v, FLEXCO_EINVAL, "NULL argument");
  const float corr1 = (float)(1.0 - pow((double)beta1, (double)step));
  const float corr2 = (float)(1.0 - pow((double)beta2, (double)step));
  hipStream_t s = (hipStream_t)stream;
  const dim3 grid((unsigned)((n + 255) / 256));
  KernelTimerScope ts(FLEXCO_K_ELEMWISE, s);
  if (dtype == FLEXCO_BF16)
    hipLaunchKernelGGL((adam_kernel<bf16_t>), grid, dim3(256), 0, s, (bf16_t*)param, master, grad, m, v, n, lr, beta1, beta2, eps, corr1, corr2);
  else
    hipLaunchKernelGGL((adam_kernel<float>), grid, dim3(256), 0, s, (float*)param, master, grad, m, v, n, lr, beta1, beta2, eps, corr1, corr2);
  return post("adam");
}
