// Fused Embedding and the core of fused multi-head attention for B models (fusion rules table rows
// "Embedding" -- one table of B*V rows, indices offset by b*V -- and "MultiheadAttention", which the
// table builds from the Linear rule: the projections are hfta_linear_fwd/bwd, and what remains is,
// per (model, sequence, head), scores = Q K^T, a row softmax, and context = P V).
//
// The three matrix products and their five adjoints are batched GEMMs over (model*sequence, head)
// on the library's GEMM core: Q, K, V are column blocks of the packed projection output
// [B][N][S][3E], addressed by leading dimension 3E and a per-head offset, so no head split or
// transpose is ever materialised; the context is written straight into its [B][N][S][E] layout.
// The softmax (scale and causal mask folded in) and its backward run in place on the score buffer,
// one wavefront per row.
#include "gemm.h"

using namespace hfta;

namespace {

// ------------------------------------------------------------------ embedding
template <typename T>
__global__ __launch_bounds__(256) void embedding_fwd_kernel(const T* __restrict__ table, const int32_t* __restrict__ idx,
                                                            const float* __restrict__ pos, T* __restrict__ out, int R,
                                                            int V, int E, int S, float scale) {
  const int r = blockIdx.x, b = blockIdx.y;
  const int v = min(max(idx[(int64_t)b * R + r], 0), V - 1);
  const T* row = table + ((int64_t)b * V + v) * E;
  T* o = out + ((int64_t)b * R + r) * E;
  const float* pr = pos ? pos + (int64_t)(r % S) * E : nullptr;
  for (int e = threadIdx.x; e < E; e += 256) Elem<T>::store(o + e, fmaf(scale, Elem<T>::load(row + e), pr ? pr[e] : 0.f));
}

__global__ __launch_bounds__(256) void zero_f32_kernel(float* __restrict__ p, int64_t n) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i + 4 <= n) *reinterpret_cast<float4*>(p + i) = make_float4(0.f, 0.f, 0.f, 0.f);
  else for (int64_t k = i; k < n; ++k) p[k] = 0.f;
}

// One workgroup per (token position p, model): if p is the first position of its table row, it lists
// the positions with the same index in increasing order (ballot + prefix counts) and adds their
// gradient rows in that order (no atomics, fixed order).
template <typename T>
__global__ __launch_bounds__(256) void embedding_bwd_kernel(const T* __restrict__ dY, const int32_t* __restrict__ idx,
                                                            float* __restrict__ dtable, int R, int V, int E, float scale) {
  extern __shared__ int32_t lidx[];                     // the model's R indices, then the list of matching positions
  __shared__ int earlier;
  __shared__ int wcnt[4];
  int32_t* match = lidx + R;
  const int p = blockIdx.x, b = blockIdx.y, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int32_t* ib = idx + (int64_t)b * R;
  for (int q = t; q < R; q += 256) lidx[q] = min(max(ib[q], 0), V - 1);
  if (t == 0) earlier = 0;
  __syncthreads();
  const int v = lidx[p];
  int found = 0;
  for (int q = t; q < p; q += 256) found |= (lidx[q] == v);
  if (found) earlier = 1;                               // benign: every writer stores 1
  __syncthreads();
  if (earlier) return;
  int total = 0;
  for (int q0 = p; q0 < R; q0 += 256) {                 // uniform trip count
    const int q = q0 + t;
    const bool hit = q < R && lidx[q] == v;
    const unsigned long long m = __ballot(hit);
    if (lane == 0) wcnt[wave] = __popcll(m);
    __syncthreads();
    int base = total;
    for (int w = 0; w < wave; ++w) base += wcnt[w];
    if (hit) match[base + __popcll(m & ((1ull << lane) - 1ull))] = q;
    total += wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
    __syncthreads();
  }
  const T* dyb = dY + (int64_t)b * R * E;
  float* dst = dtable + ((int64_t)b * V + v) * E;
  for (int e = t; e < E; e += 256) {
    float acc = 0.f;
    for (int k = 0; k < total; ++k) acc += Elem<T>::load(dyb + (int64_t)match[k] * E + e);
    dst[e] = scale * acc;
  }
}

// ------------------------------------------------------------------ softmax over score rows, in place
// rows = (batch, head, i); entry j of row i takes part if !causal or j <= i
template <typename T>
__global__ __launch_bounds__(256) void softmax_rows_kernel(T* __restrict__ P, int64_t rows, int S, float scale, int causal) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  T* p = P + row * S;
  const int lim = causal ? (int)(row % S) + 1 : S;
  float mx = -INFINITY;
  for (int j = lane; j < lim; j += 64) mx = fmaxf(mx, scale * Elem<T>::load(p + j));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  float se = 0.f;
  for (int j = lane; j < lim; j += 64) se += expf(scale * Elem<T>::load(p + j) - mx);
  se = wave_sum(se);
  const float inv = 1.f / se;
  for (int j = lane; j < S; j += 64)
    Elem<T>::store(p + j, j < lim ? expf(scale * Elem<T>::load(p + j) - mx) * inv : 0.f);
}

// dS = scale * P * (dP - sum_j dP P), in place on dP
template <typename T>
__global__ __launch_bounds__(256) void softmax_rows_bwd_kernel(const T* __restrict__ P, T* __restrict__ dP, int64_t rows,
                                                               int S, float scale) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* p = P + row * S;
  T* d = dP + row * S;
  float dot = 0.f;
  for (int j = lane; j < S; j += 64) dot = fmaf(Elem<T>::load(d + j), Elem<T>::load(p + j), dot);
  dot = wave_sum(dot);
  for (int j = lane; j < S; j += 64) {
    const float pj = Elem<T>::load(p + j);
    Elem<T>::store(d + j, scale * pj * (Elem<T>::load(d + j) - dot));
  }
}

// ------------------------------------------------------------------ softmax cross-entropy, one workgroup per row
// (wide class axes: a vocabulary).  Row loss terms go to `rowloss`; a second kernel adds them per model
// in a fixed order.
template <typename T>
__global__ __launch_bounds__(256) void xent_rows_kernel(const T* __restrict__ logits, const int32_t* __restrict__ labels,
                                                        float* __restrict__ rowloss, T* __restrict__ dlogits, int R, int K) {
  __shared__ float sh[4];
  const int r = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
  const int64_t row = (int64_t)b * R + r;
  const T* z = logits + row * K;
  T* dz = dlogits + row * K;
  auto block_max = [&](float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    __syncthreads();
    if ((t & 63) == 0) sh[t >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  };
  auto block_sum = [&](float v) {
    v = wave_sum(v);
    __syncthreads();
    if ((t & 63) == 0) sh[t >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
  };
  float mx = -INFINITY;
  for (int k = t; k < K; k += 256) mx = fmaxf(mx, Elem<T>::load(z + k));
  mx = block_max(mx);
  float se = 0.f;
  for (int k = t; k < K; k += 256) se += expf(Elem<T>::load(z + k) - mx);
  se = block_sum(se);
  const float lse = mx + logf(se);
  const int lab = labels[row];
  const float invR = 1.f / (float)R;
  for (int k = t; k < K; k += 256)
    Elem<T>::store(dz + k, (expf(Elem<T>::load(z + k) - lse) - (k == lab ? 1.f : 0.f)) * invR);
  if (t == 0) rowloss[row] = lse - Elem<T>::load(z + lab);
}

// Rows of at most 256 * NV sixteen-byte pieces (8192 bf16 / 4096 fp32 classes at NV = 4): the row
// sits in registers, so it is read once, each exponential is taken once, and the gradient leaves
// in 16-byte pieces.  Same sums as xent_rows_kernel up to fp32 summation order.
template <typename T, int NV>
__global__ __launch_bounds__(256) void xent_rows_reg_kernel(const T* __restrict__ logits, const int32_t* __restrict__ labels,
                                                            float* __restrict__ rowloss, T* __restrict__ dlogits, int R, int K) {
  constexpr int EPV = 16 / (int)sizeof(T);
  __shared__ float sh[4];
  const int r = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
  const int64_t row = (int64_t)b * R + r;
  const uint4* z = reinterpret_cast<const uint4*>(logits + row * K);
  uint4* dz = reinterpret_cast<uint4*>(dlogits + row * K);
  const int nvec = K / EPV;
  float x[NV][EPV];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int c = t + 256 * j;
    const uint4 v = c < nvec ? z[c] : make_uint4(0, 0, 0, 0);
    if constexpr (sizeof(T) == 2) {
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) { x[j][2 * i] = __uint_as_float(w[i] << 16); x[j][2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
    } else {
      x[j][0] = __uint_as_float(v.x); x[j][1] = __uint_as_float(v.y); x[j][2] = __uint_as_float(v.z); x[j][3] = __uint_as_float(v.w);
    }
#pragma unroll
    for (int e = 0; e < EPV; ++e) mx = c < nvec ? fmaxf(mx, x[j][e]) : mx;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  if ((t & 63) == 0) sh[t >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  float se = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j)
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
      x[j][e] = t + 256 * j < nvec ? __expf(x[j][e] - mx) : 0.f;     // from here on x holds exp(z - max)
      se += x[j][e];
    }
  se = wave_sum(se);
  __syncthreads();
  if ((t & 63) == 0) sh[t >> 6] = se;
  __syncthreads();
  se = (sh[0] + sh[1]) + (sh[2] + sh[3]);
  const int lab = labels[row];
  const float invR = 1.f / (float)R, inv_se = 1.f / se;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int c = t + 256 * j;
    if (c >= nvec) continue;
    float g[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) g[e] = (x[j][e] * inv_se - (c * EPV + e == lab ? 1.f : 0.f)) * invR;
    if constexpr (sizeof(T) == 2)
      dz[c] = make_uint4(pack_bf16x2(g[0], g[1]), pack_bf16x2(g[2], g[3]), pack_bf16x2(g[4], g[5]), pack_bf16x2(g[6], g[7]));
    else
      dz[c] = make_uint4(__float_as_uint(g[0]), __float_as_uint(g[1]), __float_as_uint(g[2]), __float_as_uint(g[3]));
  }
  if (t == 0) rowloss[row] = mx + logf(se) - Elem<T>::load(logits + row * K + lab);
}

__global__ __launch_bounds__(256) void xent_rows_reduce_kernel(const float* __restrict__ rowloss, float* __restrict__ loss, int R) {
  __shared__ float sh[4];
  const float* src = rowloss + (int64_t)blockIdx.x * R;
  float acc = 0.f;
  for (int i = threadIdx.x; i < R; i += 256) acc += src[i];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) loss[blockIdx.x] = ((sh[0] + sh[1]) + (sh[2] + sh[3])) / (float)R;
}

GemmDesc head_desc(int B, int N, int H, int dtype) {
  GemmDesc d{};
  d.S = 1; d.G0 = B * N; d.G1 = H;
  d.act = HFTA_ACT_NONE; d.slope = 0.f; d.dtype = dtype; d.out_f32 = false; d.splits = 1; d.partial = nullptr;
  d.bias = nullptr; d.bias_mode = 0;
  return d;
}

bool attn_ok(int B, int N, int S, int E, int H) {
  return B > 0 && N > 0 && S > 0 && E > 0 && H > 0 && E % H == 0 && (int64_t)B * N * H <= 65535;
}

}  // namespace

extern "C" {

int hfta_embedding_fwd(int B, int R, int V, int E, int dtype, const void* table, const int32_t* idx, float scale,
                       const float* pos, int S, void* out, void* stream) {
  if (B <= 0 || R <= 0 || V <= 0 || E <= 0 || !valid_dtype(dtype) || !table || !idx || !out || (pos && S <= 0)) return HFTA_EINVAL;
  if (B > 65535) return HFTA_EUNSUPPORTED;
  dim3 grid((unsigned)R, (unsigned)B);
  hipStream_t st = as_stream(stream);
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(embedding_fwd_kernel<bf16_raw>, grid, dim3(256), 0, st, (const bf16_raw*)table, idx, pos, (bf16_raw*)out,
                       R, V, E, pos ? S : 1, scale);
  else
    hipLaunchKernelGGL(embedding_fwd_kernel<float>, grid, dim3(256), 0, st, (const float*)table, idx, pos, (float*)out, R, V, E,
                       pos ? S : 1, scale);
  return launch_status();
}

int hfta_embedding_bwd(int B, int R, int V, int E, int dtype, const void* dY, const int32_t* idx, float scale,
                       float* dtable, void* stream) {
  if (B <= 0 || R <= 0 || V <= 0 || E <= 0 || !valid_dtype(dtype) || !dY || !idx || !dtable) return HFTA_EINVAL;
  if (B > 65535 || (size_t)R * 8 > 60 * 1024) return HFTA_EUNSUPPORTED;      // the model's indices and a match list are staged in LDS
  hipStream_t st = as_stream(stream);
  const int64_t n = (int64_t)B * V * E;
  hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, st, dtable, n);
  dim3 grid((unsigned)R, (unsigned)B);
  const size_t shm = (size_t)R * 8;
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(embedding_bwd_kernel<bf16_raw>, grid, dim3(256), shm, st, (const bf16_raw*)dY, idx, dtable, R, V, E, scale);
  else
    hipLaunchKernelGGL(embedding_bwd_kernel<float>, grid, dim3(256), shm, st, (const float*)dY, idx, dtable, R, V, E, scale);
  return launch_status();
}

int hfta_attention_fwd(int B, int N, int S, int E, int H, int dtype, const void* QKV, void* P, void* CTX, int causal,
                       void* stream) {
  if (!valid_dtype(dtype) || !QKV || !P || !CTX) return HFTA_EINVAL;
  if (!attn_ok(B, N, S, E, H)) return B > 0 && N > 0 && S > 0 && E > 0 && H > 0 && E % H == 0 ? HFTA_EUNSUPPORTED : HFTA_EINVAL;
  const int d = E / H;
  const size_t es = dtype_size(dtype);
  const unsigned char* q = reinterpret_cast<const unsigned char*>(QKV);
  hipStream_t st = as_stream(stream);
  const int64_t tok = (int64_t)S * 3 * E, ss = (int64_t)S * S;
  // scores[i][j] = sum_c Q[i][c] K[j][c]
  GemmDesc g = head_desc(B, N, H, dtype);
  g.A = q; g.Bm = q + (size_t)E * es; g.C = P;
  g.M = S; g.N = S; g.K = d;
  g.a_kc = true; g.a_ld = 3 * E; g.a_g0 = tok; g.a_g1 = d;
  g.b_kc = true; g.b_ld = 3 * E; g.b_g0 = tok; g.b_g1 = d;
  g.c_ld = S; g.c_g0 = (int64_t)H * ss; g.c_g1 = ss;
  int rc = gemm_launch(g, st);
  if (rc != HFTA_OK) return rc;
  const int64_t rows = (int64_t)B * N * H * S;
  const float scale = 1.f / sqrtf((float)d);
  const unsigned blocks = (unsigned)((rows + 3) / 4);
  if (dtype == HFTA_BF16) hipLaunchKernelGGL(softmax_rows_kernel<bf16_raw>, dim3(blocks), dim3(256), 0, st, (bf16_raw*)P, rows, S, scale, causal);
  else hipLaunchKernelGGL(softmax_rows_kernel<float>, dim3(blocks), dim3(256), 0, st, (float*)P, rows, S, scale, causal);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  // ctx[i][c] = sum_j P[i][j] V[j][c], written into its column block of [B][N][S][E]
  GemmDesc c = head_desc(B, N, H, dtype);
  c.A = P; c.Bm = q + (size_t)2 * E * es; c.C = CTX;
  c.M = S; c.N = d; c.K = S;
  c.a_kc = true; c.a_ld = S; c.a_g0 = (int64_t)H * ss; c.a_g1 = ss;
  c.b_kc = false; c.b_ld = 3 * E; c.b_g0 = tok; c.b_g1 = d;
  c.c_ld = E; c.c_g0 = (int64_t)S * E; c.c_g1 = d;
  return gemm_launch(c, st);
}

size_t hfta_attention_bwd_workspace_bytes(int B, int N, int S, int E, int H, int dtype) {
  if (!attn_ok(B, N, S, E, H) || !valid_dtype(dtype)) return 0;
  return (size_t)B * N * H * S * S * dtype_size(dtype);
}

int hfta_attention_bwd(int B, int N, int S, int E, int H, int dtype, const void* QKV, const void* P, const void* dCTX,
                       void* dQKV, void* workspace, size_t ws_bytes, void* stream) {
  if (!valid_dtype(dtype) || !QKV || !P || !dCTX || !dQKV) return HFTA_EINVAL;
  if (!attn_ok(B, N, S, E, H)) return B > 0 && N > 0 && S > 0 && E > 0 && H > 0 && E % H == 0 ? HFTA_EUNSUPPORTED : HFTA_EINVAL;
  if (!workspace || ws_bytes < hfta_attention_bwd_workspace_bytes(B, N, S, E, H, dtype)) return HFTA_EWORKSPACE;
  const int d = E / H;
  const size_t es = dtype_size(dtype);
  const unsigned char* q = reinterpret_cast<const unsigned char*>(QKV);
  unsigned char* dq = reinterpret_cast<unsigned char*>(dQKV);
  hipStream_t st = as_stream(stream);
  const int64_t tok = (int64_t)S * 3 * E, ss = (int64_t)S * S, hs = (int64_t)H * ss;
  // dV[j][c] = sum_i P[i][j] dCTX[i][c]
  GemmDesc g = head_desc(B, N, H, dtype);
  g.A = P; g.Bm = dCTX; g.C = dq + (size_t)2 * E * es;
  g.M = S; g.N = d; g.K = S;
  g.a_kc = false; g.a_ld = S; g.a_g0 = hs; g.a_g1 = ss;
  g.b_kc = false; g.b_ld = E; g.b_g0 = (int64_t)S * E; g.b_g1 = d;
  g.c_ld = 3 * E; g.c_g0 = tok; g.c_g1 = d;
  int rc = gemm_launch(g, st);
  if (rc != HFTA_OK) return rc;
  // dP[i][j] = sum_c dCTX[i][c] V[j][c]
  g = head_desc(B, N, H, dtype);
  g.A = dCTX; g.Bm = q + (size_t)2 * E * es; g.C = workspace;
  g.M = S; g.N = S; g.K = d;
  g.a_kc = true; g.a_ld = E; g.a_g0 = (int64_t)S * E; g.a_g1 = d;
  g.b_kc = true; g.b_ld = 3 * E; g.b_g0 = tok; g.b_g1 = d;
  g.c_ld = S; g.c_g0 = hs; g.c_g1 = ss;
  rc = gemm_launch(g, st);
  if (rc != HFTA_OK) return rc;
  const int64_t rows = (int64_t)B * N * H * S;
  const float scale = 1.f / sqrtf((float)d);
  const unsigned blocks = (unsigned)((rows + 3) / 4);
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(softmax_rows_bwd_kernel<bf16_raw>, dim3(blocks), dim3(256), 0, st, (const bf16_raw*)P, (bf16_raw*)workspace, rows, S, scale);
  else
    hipLaunchKernelGGL(softmax_rows_bwd_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)P, (float*)workspace, rows, S, scale);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  // dQ[i][c] = sum_j dS[i][j] K[j][c]
  g = head_desc(B, N, H, dtype);
  g.A = workspace; g.Bm = q + (size_t)E * es; g.C = dq;
  g.M = S; g.N = d; g.K = S;
  g.a_kc = true; g.a_ld = S; g.a_g0 = hs; g.a_g1 = ss;
  g.b_kc = false; g.b_ld = 3 * E; g.b_g0 = tok; g.b_g1 = d;
  g.c_ld = 3 * E; g.c_g0 = tok; g.c_g1 = d;
  rc = gemm_launch(g, st);
  if (rc != HFTA_OK) return rc;
  // dK[j][c] = sum_i dS[i][j] Q[i][c]
  g = head_desc(B, N, H, dtype);
  g.A = workspace; g.Bm = q; g.C = dq + (size_t)E * es;
  g.M = S; g.N = d; g.K = S;
  g.a_kc = false; g.a_ld = S; g.a_g0 = hs; g.a_g1 = ss;
  g.b_kc = false; g.b_ld = 3 * E; g.b_g0 = tok; g.b_g1 = d;
  g.c_ld = 3 * E; g.c_g0 = tok; g.c_g1 = d;
  return gemm_launch(g, st);
}

size_t hfta_softmax_xent_rows_workspace_bytes(int B, int R) {
  if (B <= 0 || R <= 0) return 0;
  return (size_t)B * R * sizeof(float);
}

int hfta_softmax_xent_rows(int B, int R, int K, int dtype, const void* logits, const int32_t* labels, float* loss,
                           void* dlogits, void* workspace, size_t ws_bytes, void* stream) {
  if (B <= 0 || R <= 0 || K <= 0 || !valid_dtype(dtype) || !logits || !labels || !loss || !dlogits) return HFTA_EINVAL;
  if (B > 65535) return HFTA_EUNSUPPORTED;
  if (!workspace || ws_bytes < hfta_softmax_xent_rows_workspace_bytes(B, R)) return HFTA_EWORKSPACE;
  hipStream_t st = as_stream(stream);
  dim3 grid((unsigned)R, (unsigned)B);
  const int epv = 16 / (int)dtype_size(dtype);
  const bool in_regs = K % epv == 0 && K / epv <= 256 * 4 && reinterpret_cast<uintptr_t>(logits) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(dlogits) % 16 == 0;
  if (in_regs && dtype == HFTA_BF16)
    hipLaunchKernelGGL((xent_rows_reg_kernel<bf16_raw, 4>), grid, dim3(256), 0, st, (const bf16_raw*)logits, labels,
                       (float*)workspace, (bf16_raw*)dlogits, R, K);
  else if (in_regs)
    hipLaunchKernelGGL((xent_rows_reg_kernel<float, 4>), grid, dim3(256), 0, st, (const float*)logits, labels,
                       (float*)workspace, (float*)dlogits, R, K);
  else if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(xent_rows_kernel<bf16_raw>, grid, dim3(256), 0, st, (const bf16_raw*)logits, labels, (float*)workspace,
                       (bf16_raw*)dlogits, R, K);
  else
    hipLaunchKernelGGL(xent_rows_kernel<float>, grid, dim3(256), 0, st, (const float*)logits, labels, (float*)workspace,
                       (float*)dlogits, R, K);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  hipLaunchKernelGGL(xent_rows_reduce_kernel, dim3((unsigned)B), dim3(256), 0, st, (const float*)workspace, loss, R);
  return launch_status();
}

// Per-sample point transform (the point-cloud models' input / feature transform): the weight of this
// k=1 convolution is indexed by the sample as well as by the model, T:[B][Nb][Co][Ci].
int hfta_point_transform_fwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                             const void* T, void* Y, const int64_t ys[4], void* stream) {
  if (B <= 0 || Nb <= 0 || Ci <= 0 || Co <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !T || !Y || !ys) return HFTA_EINVAL;
  if (xs[3] != 1 || ys[3] != 1 || (int64_t)B * Nb > 65535) return HFTA_EUNSUPPORTED;
  GemmDesc g = head_desc(B, 1, Nb, dtype);
  g.A = T; g.Bm = X; g.C = Y;
  g.M = Co; g.N = L; g.K = Ci;
  g.a_kc = true; g.a_ld = Ci; g.a_g0 = (int64_t)Nb * Co * Ci; g.a_g1 = (int64_t)Co * Ci;
  g.b_kc = false; g.b_ld = xs[2]; g.b_g0 = xs[0]; g.b_g1 = xs[1];
  g.c_ld = ys[2]; g.c_g0 = ys[0]; g.c_g1 = ys[1];
  return gemm_launch(g, as_stream(stream));
}

int hfta_point_transform_bwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                             const void* T, const void* dY, const int64_t dys[4], void* dX, const int64_t dxs[4],
                             void* dT, void* stream) {
  if (B <= 0 || Nb <= 0 || Ci <= 0 || Co <= 0 || L <= 0 || !valid_dtype(dtype) || !dY || !dys) return HFTA_EINVAL;
  if ((dX && (!T || !dxs)) || (dT && (!X || !xs))) return HFTA_EINVAL;
  if (dys[3] != 1 || (dX && dxs[3] != 1) || (dT && xs[3] != 1) || (int64_t)B * Nb > 65535) return HFTA_EUNSUPPORTED;
  hipStream_t st = as_stream(stream);
  if (dX) {      // dX[c][l] = sum_o T[o][c] dY[o][l]
    GemmDesc g = head_desc(B, 1, Nb, dtype);
    g.A = T; g.Bm = dY; g.C = dX;
    g.M = Ci; g.N = L; g.K = Co;
    g.a_kc = false; g.a_ld = Ci; g.a_g0 = (int64_t)Nb * Co * Ci; g.a_g1 = (int64_t)Co * Ci;
    g.b_kc = false; g.b_ld = dys[2]; g.b_g0 = dys[0]; g.b_g1 = dys[1];
    g.c_ld = dxs[2]; g.c_g0 = dxs[0]; g.c_g1 = dxs[1];
    const int rc = gemm_launch(g, st);
    if (rc != HFTA_OK) return rc;
  }
  if (dT) {      // dT[o][c] = sum_l dY[o][l] X[c][l], per sample: no reduction over the batch
    GemmDesc g = head_desc(B, 1, Nb, dtype);
    g.A = dY; g.Bm = X; g.C = dT;
    g.M = Co; g.N = Ci; g.K = L;
    g.a_kc = true; g.a_ld = dys[2]; g.a_g0 = dys[0]; g.a_g1 = dys[1];
    g.b_kc = true; g.b_ld = xs[2]; g.b_g0 = xs[0]; g.b_g1 = xs[1];
    g.c_ld = Ci; g.c_g0 = (int64_t)Nb * Co * Ci; g.c_g1 = (int64_t)Co * Ci;
    return gemm_launch(g, st);
  }
  return HFTA_OK;
}

}  // extern "C"
