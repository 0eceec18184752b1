// Shape-generic HIP kernels of the decoder stage: the fp32 path runs entirely on these,
// and the bf16 path uses them for every shape its MFMA kernels do not cover.
// Operator definitions: Llama-2 pre-norm decoder block (the layer arithmetic that the
// paper's Section 6 adopts from Meta's Llama inference code).
#include "kernels.hpp"
#include "device_util.hpp"

namespace ls {

// ------------------------------------------------------------------ row bookkeeping
__global__ void k_row_index_prefill(const int32_t* __restrict__ cu, int batch, int total,
                                    int32_t* row_seq, int32_t* row_pos, int32_t* last_rows) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < batch) last_rows[t] = cu[t + 1] - 1;
  if (t >= total) return;
  int lo = 0, hi = batch;  // find b with cu[b] <= t < cu[b+1]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  row_seq[t] = lo;
  row_pos[t] = t - cu[lo];
}

__global__ void k_row_index_decode(const int32_t* __restrict__ seq_lens, int batch, int max_seq,
                                   int32_t* row_seq, int32_t* row_pos, int32_t* last_rows) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  int p = seq_lens[b];
  row_seq[b] = b;
  row_pos[b] = (p >= 0 && p < max_seq) ? p : -1;
  last_rows[b] = b;
}

__global__ void k_seq_lens_set(const int32_t* __restrict__ cu, int batch, int32_t* seq_lens) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < batch) seq_lens[b] = cu[b + 1] - cu[b];
}

__global__ void k_seq_lens_inc(int batch, int max_seq, int32_t* seq_lens) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < batch && seq_lens[b] >= 0 && seq_lens[b] < max_seq) seq_lens[b] += 1;
}

// One decode step's bookkeeping and first-layer inputs in a single launch, one workgroup
// per sequence: row maps, seq_lens += 1 (a full sequence is left alone and marked -1), the
// fp32 residual row, its bf16 copy, and the sum of squares of every 16-column tile.
template <class T>
__global__ void __launch_bounds__(256) k_decode_prologue(const T* __restrict__ table, const void* __restrict__ in,
                                                         int32_t* seq_lens, int max_seq, int d, int vocab,
                                                         int32_t* row_seq, int32_t* row_pos, int32_t* last_rows,
                                                         float* __restrict__ x, T* __restrict__ xb,
                                                         float* __restrict__ ss_part, const T* __restrict__ gamma) {
  const int b = blockIdx.x;
  if (threadIdx.x == 0) {
    const int p = seq_lens[b];
    const bool ok = p >= 0 && p < max_seq;
    row_seq[b] = b;
    row_pos[b] = ok ? p : -1;
    last_rows[b] = b;
    if (ok) seq_lens[b] = p + 1;
  }
  const T* src;
  if (table) {
    int id = ((const int32_t*)in)[b];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    src = table + (size_t)id * d;
  } else {
    src = (const T*)in + (size_t)b * d;
  }
  // 16-byte accesses when the element is bf16 and the input row is 16-byte aligned (the
  // workspace rows and the weight slab always are); same arithmetic, same summation order
  bool vec = false;
  if constexpr (sizeof(T) == 2) vec = ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(gamma)) & 15) == 0;
  for (int tile = threadIdx.x; tile < (d >> 4); tile += 256) {
    float ss = 0.f;
    const size_t o = (size_t)b * d + tile * 16;
    if constexpr (sizeof(T) == 2) {
      if (vec) {
        bf16x8 raw[2], g[2], y[2];
        raw[0] = *reinterpret_cast<const bf16x8*>(src + tile * 16);
        raw[1] = *reinterpret_cast<const bf16x8*>(src + tile * 16 + 8);
        if (gamma) {
          g[0] = *reinterpret_cast<const bf16x8*>(gamma + tile * 16);
          g[1] = *reinterpret_cast<const bf16x8*>(gamma + tile * 16 + 8);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          f32x4 lo, hi;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float v = (float)raw[h][e];
            if (e < 4) lo[e] = v; else hi[e - 4] = v;
            y[h][e] = gamma ? (bf16)(v * (float)g[h][e]) : raw[h][e];
            ss += v * v;
          }
          *reinterpret_cast<f32x4*>(x + o + h * 8) = lo;
          *reinterpret_cast<f32x4*>(x + o + h * 8 + 4) = hi;
          *reinterpret_cast<bf16x8*>(xb + o + h * 8) = y[h];
        }
        ss_part[(size_t)b * (d >> 4) + tile] = ss;
        continue;
      }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const T raw = src[tile * 16 + e];
      const float v = to_f(raw);
      x[o + e] = v;
      xb[o + e] = gamma ? from_f<T>(v * to_f(gamma[tile * 16 + e])) : raw;
      ss += v * v;
    }
    ss_part[(size_t)b * (d >> 4) + tile] = ss;
  }
}

void launch_decode_prologue(uint32_t dt, const void* table, const void* in, int32_t* seq_lens, int batch, int max_seq,
                            int d, int vocab, int32_t* row_seq, int32_t* row_pos, int32_t* last_rows, float* x,
                            void* xb, float* ss_part, const void* gamma, hipStream_t st) {
  if (dt == F32)
    k_decode_prologue<float><<<batch, 256, 0, st>>>((const float*)table, in, seq_lens, max_seq, d, vocab, row_seq,
                                                    row_pos, last_rows, x, (float*)xb, ss_part, (const float*)gamma);
  else
    k_decode_prologue<bf16><<<batch, 256, 0, st>>>((const bf16*)table, in, seq_lens, max_seq, d, vocab, row_seq,
                                                   row_pos, last_rows, x, (bf16*)xb, ss_part, (const bf16*)gamma);
}

void launch_row_index_prefill(const int32_t* cu, int batch, int total, int32_t* row_seq,
                              int32_t* row_pos, int32_t* last_rows, hipStream_t st) {
  int n = total > batch ? total : batch;
  k_row_index_prefill<<<(n + 255) / 256, 256, 0, st>>>(cu, batch, total, row_seq, row_pos, last_rows);
}
void launch_row_index_decode(const int32_t* seq_lens, int batch, int max_seq, int32_t* row_seq,
                             int32_t* row_pos, int32_t* last_rows, hipStream_t st) {
  k_row_index_decode<<<(batch + 255) / 256, 256, 0, st>>>(seq_lens, batch, max_seq, row_seq, row_pos, last_rows);
}
void launch_seq_lens_set(const int32_t* cu, int batch, int32_t* seq_lens, hipStream_t st) {
  k_seq_lens_set<<<(batch + 255) / 256, 256, 0, st>>>(cu, batch, seq_lens);
}
void launch_seq_lens_inc(int batch, int max_seq, int32_t* seq_lens, hipStream_t st) {
  k_seq_lens_inc<<<(batch + 255) / 256, 256, 0, st>>>(batch, max_seq, seq_lens);
}

// ------------------------------------------------------------------ stage input / output
template <class T>
__global__ void k_embed(const T* __restrict__ table, const int32_t* __restrict__ tok, float* x,
                        int rows, int d, int vocab) {
  int r = blockIdx.x;
  int id = tok[r];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);  // an id outside the table is clamped
  const T* src = table + (size_t)id * d;
  float* dst = x + (size_t)r * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = to_f(src[i]);
}

template <class T>
__global__ void k_load_hidden(const T* __restrict__ in, float* x, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) x[i] = to_f(in[i]);
}

template <class T>
__global__ void k_store_hidden(const float* __restrict__ x, T* out, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = from_f<T>(x[i]);
}

void launch_embed(uint32_t dt, const void* table, const int32_t* tok, float* x, int rows, int d,
                  int vocab, hipStream_t st) {
  if (rows <= 0) return;
  if (dt == F32) k_embed<float><<<rows, 256, 0, st>>>((const float*)table, tok, x, rows, d, vocab);
  else k_embed<bf16><<<rows, 256, 0, st>>>((const bf16*)table, tok, x, rows, d, vocab);
}
static inline int grid_for(size_t n) {
  size_t g = (n + 255) / 256;
  return (int)(g > 65536 ? 65536 : (g ? g : 1));
}
void launch_load_hidden(uint32_t dt, const void* in, float* x, size_t n, hipStream_t st) {
  if (!n) return;
  if (dt == F32) k_load_hidden<float><<<grid_for(n), 256, 0, st>>>((const float*)in, x, n);
  else k_load_hidden<bf16><<<grid_for(n), 256, 0, st>>>((const bf16*)in, x, n);
}
void launch_store_hidden(uint32_t dt, const float* x, void* out, size_t n, hipStream_t st) {
  if (!n) return;
  if (dt == F32) k_store_hidden<float><<<grid_for(n), 256, 0, st>>>(x, (float*)out, n);
  else k_store_hidden<bf16><<<grid_for(n), 256, 0, st>>>(x, (bf16*)out, n);
}

// ------------------------------------------------------------------ RMSNorm
// One 256-thread workgroup per row; the sum of squares is reduced in a fixed order
// (lane tree, then the four wave partials in index order), so results are reproducible.
template <class T>
__global__ void __launch_bounds__(256) k_rmsnorm(const float* __restrict__ x, const T* __restrict__ gamma,
                                                 T* __restrict__ y, int d, float eps,
                                                 const int32_t* __restrict__ row_map) {
  __shared__ float part[4];
  int r = blockIdx.x;
  const float* xr = x + (size_t)(row_map ? row_map[r] : r) * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) { float v = xr[i]; ss += v * v; }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = (part[0] + part[1]) + (part[2] + part[3]);
  float inv = 1.0f / sqrtf(tot / (float)d + eps);
  T* yr = y + (size_t)r * d;
  for (int i = threadIdx.x; i < d; i += 256) yr[i] = from_f<T>(xr[i] * inv * to_f(gamma[i]));
}

// Fast path for d % 4 == 0 and d <= 8192: the row lives in registers (up to eight 16-byte
// loads per thread, all issued before the first use), so x is read exactly once.
template <class T>
__global__ void __launch_bounds__(256) k_rmsnorm_vec(const float* __restrict__ x, const T* __restrict__ gamma,
                                                     T* __restrict__ y, int d, float eps,
                                                     const int32_t* __restrict__ row_map) {
  __shared__ float part[4];
  const int r = blockIdx.x, nv = d >> 2;
  const f32x4* xr = reinterpret_cast<const f32x4*>(x + (size_t)(row_map ? row_map[r] : r) * d);
  f32x4 v[8];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int idx = threadIdx.x + 256 * i;
    v[i] = idx < nv ? xr[idx] : f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) ss += v[i][0] * v[i][0] + v[i][1] * v[i][1] + v[i][2] * v[i][2] + v[i][3] * v[i][3];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = (part[0] + part[1]) + (part[2] + part[3]);
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  T* yr = y + (size_t)r * d;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int idx = threadIdx.x + 256 * i;
    if (idx < nv) {
#pragma unroll
      for (int e = 0; e < 4; ++e) yr[idx * 4 + e] = from_f<T>(v[i][e] * inv * to_f(gamma[idx * 4 + e]));
    }
  }
}

void launch_rmsnorm(uint32_t dt, const float* x, const void* gamma, void* y, int rows, int d,
                    float eps, const int32_t* row_map, hipStream_t st) {
  if (rows <= 0) return;
  const bool vec = (d % 4 == 0) && d <= 8192;
  if (dt == F32) {
    if (vec) k_rmsnorm_vec<float><<<rows, 256, 0, st>>>(x, (const float*)gamma, (float*)y, d, eps, row_map);
    else k_rmsnorm<float><<<rows, 256, 0, st>>>(x, (const float*)gamma, (float*)y, d, eps, row_map);
  } else {
    if (vec) k_rmsnorm_vec<bf16><<<rows, 256, 0, st>>>(x, (const bf16*)gamma, (bf16*)y, d, eps, row_map);
    else k_rmsnorm<bf16><<<rows, 256, 0, st>>>(x, (const bf16*)gamma, (bf16*)y, d, eps, row_map);
  }
}

// ------------------------------------------------------------------ generic GEMM
// C[M,N] = A[M,K] W[N,K]^T.  64x64 tile per 256-thread workgroup, 4x4 outputs per thread,
// fp32 FMAs from LDS.  Any M, N, K.
template <class T, int EPI>
__global__ void __launch_bounds__(256) k_gemm_generic(const T* __restrict__ A, const T* __restrict__ W,
                                                      int M, int N, int K, void* __restrict__ outv,
                                                      float* __restrict__ resid) {
  constexpr int BM = 64, BN = 64, BK = 16, PAD = 4;
  constexpr bool GLU = (EPI == EPI_SWIGLU);
  __shared__ float As[BK][BM + PAD];
  __shared__ float Ws[BK][BN + PAD];
  __shared__ float Us[GLU ? BK : 1][BN + PAD];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int lr = tid >> 2, lk = (tid & 3) * 4;  // loader: row lr, 4 consecutive k
  float acc[4][4] = {}, accu[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int k = k0 + lk + j;
      int am = m0 + lr, wn = n0 + lr;
      As[lk + j][lr] = (am < M && k < K) ? to_f(A[(size_t)am * K + k]) : 0.f;
      Ws[lk + j][lr] = (wn < N && k < K) ? to_f(W[(size_t)wn * K + k]) : 0.f;
      if constexpr (GLU) Us[lk + j][lr] = (wn < N && k < K) ? to_f(W[((size_t)N + wn) * K + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], w[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; w[i] = Ws[k][tx * 4 + i]; }
      if constexpr (GLU) {
#pragma unroll
        for (int i = 0; i < 4; ++i) u[i] = Us[k][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
          if constexpr (GLU) accu[i][j] = fmaf(a[i], u[j], accu[i][j]);
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      size_t o = (size_t)m * N + n;
      if constexpr (EPI == EPI_STORE) ((T*)outv)[o] = from_f<T>(acc[i][j]);
      else if constexpr (EPI == EPI_RESID) resid[o] += acc[i][j];
      else if constexpr (EPI == EPI_SWIGLU) ((T*)outv)[o] = from_f<T>(silu_f(acc[i][j]) * accu[i][j]);
      else ((float*)outv)[o] = acc[i][j];
    }
  }
}

template <class T>
static void gemm_generic_t(Epilogue epi, const void* A, const void* W, int M, int N, int K, void* out,
                           float* resid, hipStream_t st) {
  dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
  const T* a = (const T*)A; const T* w = (const T*)W;
  switch (epi) {
    case EPI_STORE: k_gemm_generic<T, EPI_STORE><<<grid, block, 0, st>>>(a, w, M, N, K, out, resid); break;
    case EPI_RESID: k_gemm_generic<T, EPI_RESID><<<grid, block, 0, st>>>(a, w, M, N, K, out, resid); break;
    case EPI_SWIGLU: k_gemm_generic<T, EPI_SWIGLU><<<grid, block, 0, st>>>(a, w, M, N, K, out, resid); break;
    case EPI_F32: k_gemm_generic<T, EPI_F32><<<grid, block, 0, st>>>(a, w, M, N, K, out, resid); break;
  }
}

void launch_gemm_generic(uint32_t dt, Epilogue epi, const void* A, const void* W, int M, int N, int K,
                         void* out, float* resid, hipStream_t st) {
  if (M <= 0 || N <= 0) return;
  if (dt == F32) gemm_generic_t<float>(epi, A, W, M, N, K, out, resid, st);
  else gemm_generic_t<bf16>(epi, A, W, M, N, K, out, resid, st);
}

// ------------------------------------------------------------------ RoPE + KV append
// One workgroup per row.  Pair i of a head is (2i, 2i+1); it turns by the angle whose
// cosine and sine sit in cs[pos][i].  q is rotated in place, k is rotated into the cache,
// v is copied into the cache.
template <class T>
__global__ void __launch_bounds__(256) k_rope_append(T* __restrict__ qkv, const float2* __restrict__ cs,
                                                     const int32_t* __restrict__ row_seq,
                                                     const int32_t* __restrict__ row_pos, int hq, int hkv,
                                                     int hd, int max_seq, T* __restrict__ kc, T* __restrict__ vc) {
  int r = blockIdx.x;
  int pos = row_pos[r];
  if (pos < 0) return;
  int seq = row_seq[r];
  int half = hd >> 1;
  int npairs = (hq + 2 * hkv) * half;
  T* row = qkv + (size_t)r * (hq + 2 * hkv) * hd;
  for (int p = threadIdx.x; p < npairs; p += 256) {
    int head = p / half, i = p - head * half;
    T* src = row + (size_t)head * hd + 2 * i;
    float u0 = to_f(src[0]), u1 = to_f(src[1]);
    if (head < hq + hkv) {
      float2 c = cs[(size_t)pos * half + i];
      float r0 = u0 * c.x - u1 * c.y, r1 = u0 * c.y + u1 * c.x;
      u0 = r0; u1 = r1;
    }
    if (head < hq) {
      src[0] = from_f<T>(u0); src[1] = from_f<T>(u1);
    } else {
      bool isv = head >= hq + hkv;
      int kh = isv ? head - hq - hkv : head - hq;
      size_t o = (((size_t)seq * hkv + kh) * max_seq + pos) * hd + 2 * i;
      T* dst = (isv ? vc : kc) + o;
      dst[0] = from_f<T>(u0); dst[1] = from_f<T>(u1);
    }
  }
}

// bf16 fast path (head_dim % 8 == 0): a thread owns 8 consecutive elements (4 pairs) of one
// head of one row: one 16-byte load, two 16-byte table loads, one 16-byte store.
__global__ void __launch_bounds__(256) k_rope_append_vec(bf16* __restrict__ qkv, const float* __restrict__ cs,
                                                         const int32_t* __restrict__ row_seq,
                                                         const int32_t* __restrict__ row_pos, int hq, int hkv,
                                                         int hd, int max_seq, bf16* __restrict__ kc,
                                                         bf16* __restrict__ vc) {
  const int r = blockIdx.x;
  const int pos = row_pos[r];
  if (pos < 0) return;
  const int cpr = hd >> 3;                       // 16-byte chunks per head
  const int item = blockIdx.y * 256 + threadIdx.x;
  if (item >= (hq + 2 * hkv) * cpr) return;
  const int head = item / cpr, ch = item - head * cpr;
  bf16* src = qkv + (size_t)r * (hq + 2 * hkv) * hd + (size_t)head * hd + ch * 8;
  bf16x8 v = *reinterpret_cast<const bf16x8*>(src);
  if (head < hq + hkv) {
    const f32x4* t = reinterpret_cast<const f32x4*>(cs + ((size_t)pos * (hd >> 1) + ch * 4) * 2);
    const f32x4 t0 = t[0], t1 = t[1];  // (cos, sin) of pairs 0,1 and 2,3
    const float c[4] = {t0[0], t0[2], t1[0], t1[2]}, sn[4] = {t0[1], t0[3], t1[1], t1[3]};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float u0 = (float)v[2 * i], u1 = (float)v[2 * i + 1];
      v[2 * i] = (bf16)(u0 * c[i] - u1 * sn[i]);
      v[2 * i + 1] = (bf16)(u0 * sn[i] + u1 * c[i]);
    }
  }
  if (head < hq) {
    *reinterpret_cast<bf16x8*>(src) = v;
  } else {
    const bool isv = head >= hq + hkv;
    const int kh = isv ? head - hq - hkv : head - hq;
    const size_t o = (((size_t)row_seq[r] * hkv + kh) * max_seq + pos) * hd + ch * 8;
    *reinterpret_cast<bf16x8*>((isv ? vc : kc) + o) = v;
  }
}

void launch_rope_append(uint32_t dt, void* qkv, const float* cs_table, const int32_t* row_seq,
                        const int32_t* row_pos, int rows, int hq, int hkv, int hd, int max_seq,
                        void* kcache, void* vcache, hipStream_t st) {
  if (rows <= 0) return;
  if (dt == F32)
    k_rope_append<float><<<rows, 256, 0, st>>>((float*)qkv, (const float2*)cs_table, row_seq, row_pos, hq, hkv,
                                               hd, max_seq, (float*)kcache, (float*)vcache);
  else if (hd % 8 == 0) {
    dim3 grid(rows, ((hq + 2 * hkv) * (hd / 8) + 255) / 256);
    k_rope_append_vec<<<grid, 256, 0, st>>>((bf16*)qkv, cs_table, row_seq, row_pos, hq, hkv, hd, max_seq,
                                            (bf16*)kcache, (bf16*)vcache);
  } else
    k_rope_append<bf16><<<rows, 256, 0, st>>>((bf16*)qkv, (const float2*)cs_table, row_seq, row_pos, hq, hkv,
                                              hd, max_seq, (bf16*)kcache, (bf16*)vcache);
}

// ------------------------------------------------------------------ generic attention
// One wavefront per (row, query head): the lanes split head_dim, keys are visited in
// order with a running maximum and running sum (online softmax), all in fp32.
template <class T>
__global__ void __launch_bounds__(64) k_attention_generic(const T* __restrict__ qkv, int qkv_stride,
                                                          const T* __restrict__ kc, const T* __restrict__ vc,
                                                          const int32_t* __restrict__ row_seq,
                                                          const int32_t* __restrict__ row_pos, int hq, int hkv,
                                                          int hd, int max_seq, T* __restrict__ out) {
  constexpr int MAXI = 4;  // head_dim <= 256
  int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  int pos = row_pos[r];
  if (pos < 0) return;
  int seq = row_seq[r];
  int kh = h / (hq / hkv);
  const T* q = qkv + (size_t)r * qkv_stride + (size_t)h * hd;
  const T* kb = kc + ((size_t)seq * hkv + kh) * max_seq * hd;
  const T* vb = vc + ((size_t)seq * hkv + kh) * max_seq * hd;
  float scale = 1.0f / sqrtf((float)hd);
  float qv[MAXI], acc[MAXI];
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    int e = lane + 64 * i;
    qv[i] = e < hd ? to_f(q[e]) * scale : 0.f;
    acc[i] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  for (int j = 0; j <= pos; ++j) {
    const T* kr = kb + (size_t)j * hd;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      int e = lane + 64 * i;
      if (e < hd) s = fmaf(qv[i], to_f(kr[e]), s);
    }
    s = wave_sum(s);
    float mn = fmaxf(m, s);
    float corr = __expf(m - mn), p = __expf(s - mn);
    l = l * corr + p;
    const T* vr = vb + (size_t)j * hd;
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      int e = lane + 64 * i;
      if (e < hd) acc[i] = acc[i] * corr + p * to_f(vr[e]);
    }
    m = mn;
  }
  float inv = 1.0f / l;
  T* o = out + (size_t)r * hq * hd + (size_t)h * hd;
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    int e = lane + 64 * i;
    if (e < hd) o[e] = from_f<T>(acc[i] * inv);
  }
}

void launch_attention_generic(uint32_t dt, const void* qkv, int qkv_stride, const void* kcache,
                              const void* vcache, const int32_t* row_seq, const int32_t* row_pos, int rows,
                              int hq, int hkv, int hd, int max_seq, void* out, hipStream_t st) {
  if (rows <= 0) return;
  dim3 grid(rows, hq);
  if (dt == F32)
    k_attention_generic<float><<<grid, 64, 0, st>>>((const float*)qkv, qkv_stride, (const float*)kcache,
                                                    (const float*)vcache, row_seq, row_pos, hq, hkv, hd, max_seq,
                                                    (float*)out);
  else
    k_attention_generic<bf16><<<grid, 64, 0, st>>>((const bf16*)qkv, qkv_stride, (const bf16*)kcache,
                                                   (const bf16*)vcache, row_seq, row_pos, hq, hkv, hd, max_seq,
                                                   (bf16*)out);
}

// ------------------------------------------------------------------ greedy argmax
// One 1024-thread workgroup per row.  A thread walks its indices in ascending order, eight
// independent loads at a time (one memory round trip per eight elements instead of per element).
__global__ void __launch_bounds__(1024) k_argmax(const float* __restrict__ logits, int vocab, int32_t* tok) {
  constexpr int NT = 1024, U = 8;
  __shared__ float bv[NT / 64];
  __shared__ int bi[NT / 64];
  const float* row = logits + (size_t)blockIdx.x * vocab;
  float best = -INFINITY;
  int idx = 0x7fffffff;
  for (int i0 = threadIdx.x; i0 < vocab; i0 += NT * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * NT;
      v[u] = i < vocab ? row[i] : -INFINITY;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * NT;
      if (i < vocab && (v[u] > best || idx == 0x7fffffff)) { best = v[u]; idx = i; }  // ascending i: ties keep the lower index
    }
  }
  for (int off = 32; off; off >>= 1) {
    float ov = __shfl_xor(best, off);
    int oi = __shfl_xor(idx, off);
    if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
  }
  if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = idx; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < NT / 64; ++w)
      if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
    tok[blockIdx.x] = idx;
  }
}

void launch_argmax(const float* logits, int rows, int vocab, int32_t* tok, hipStream_t st) {
  if (rows <= 0) return;
  k_argmax<<<rows, 1024, 0, st>>>(logits, vocab, tok);
}

}  // namespace ls
