// bf16 weight-streaming GEMM for decode steps: C[M,N] = X[M,K] W[N,K]^T with M <= 64.
//
// At M <= 64 every weight byte is used for at most 64 multiply-adds, so the kernel is bound
// by how fast W streams out of HBM (roofline: HBM bandwidth), and the design goal is to read
// each byte of W exactly once with fully used cache lines and many bytes in flight.
//
//   * A workgroup owns 16 output columns (16 rows of W; with the SwiGLU epilogue, the 16
//     gate rows and the 16 up rows of the same columns).  Its KS wavefronts split K.
//   * A wavefront walks its K range in blocks of 128: four 16-byte-per-lane global loads
//     fetch 16 rows x 256 contiguous bytes (a quarter-wave per row, whole cache lines), held
//     in a register ring several blocks deep so that >= 8 KB per wave is always in flight.
//   * Each block passes through a wave-private 4 KB LDS scratch (written lane-linear, chunks
//     XOR-swizzled by row) to reach the MFMA operand layout: v_mfma_f32_16x16x32_bf16 with
//     W as the A operand (row = lane%16, 8 k-values per lane) and X as the B operand
//     (column m = lane%16); a lane of the result holds m = lane%16, n = 4*(lane/16) + r.
//   * The KS partial tiles are summed through LDS in wave order (fixed order: results are
//     reproducible), then the epilogue stores, adds to the residual stream, or applies SwiGLU.
//
// Decode-step fusion of the RMSNorms (no separate norm launches):
//   * a residual-add epilogue can also emit xb = bf16(x) and, per row and 16-column tile,
//     the sum of squares of the new x (fp32, fixed-order reduction);
//     the copy it emits is already multiplied by the gain of the norm that follows;
//   * a NORM consumer takes that copy and those partial sums instead of a normalised input
//     and scales the accumulator by 1/sqrt(mean(x^2)+eps) of its row in the epilogue.  The
//     partial sums are requested before the weight stream is walked and only added up after
//     it, so their latency hides behind the stream.
#include "kernels.hpp"
#include "device_util.hpp"

namespace ls {

namespace {

#ifndef LS_SKINNY_MINWG
#define LS_SKINNY_MINWG 1
#endif
template <int MT, int EPI, int KS, int PF, bool NORM>
__global__ void __launch_bounds__(KS * 64, LS_SKINNY_MINWG)
k_gemm_skinny(const bf16* __restrict__ X, const bf16* __restrict__ W, int M, int N, int K,
              void* __restrict__ outv, float* __restrict__ resid, SkinnyFusion fu) {
  constexpr bool GLU = (EPI == EPI_SWIGLU);
  constexpr int NW = GLU ? 2 : 1;                      // weight streams per wave
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float sm_inv[MT * 16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int n0 = blockIdx.x * 16;
  const int nblk = K >> 7;
  const int b0 = (int)((long)wave * nblk / KS), b1 = (int)((long)(wave + 1) * nblk / KS);
  const int nb = b1 - b0;
  unsigned char* scratch = smem + wave * (NW * 4096);
  // per-lane global offsets (elements) of the four load instructions of a block
  size_t woff[NW][4];
#pragma unroll
  for (int s = 0; s < NW; ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 4 * i + lg;
      woff[s][i] = (size_t)(s * N + n0 + row) * K + (size_t)((lr ^ row) << 3);
    }
  u32x4 wr[PF][NW][4];
  // weights are read exactly once per launch: non-temporal loads keep them from displacing
  // the activations in the caches and stream measurably faster out of HBM
#ifndef LS_STREAM_LOAD
#define LS_STREAM_LOAD(p) __builtin_nontemporal_load(p)
#endif
#define LS_LOAD_W(slot, blk)                                                                     \
  {                                                                                              \
    const size_t kb_ = (size_t)(blk) << 7;                                                       \
    _Pragma("unroll") for (int s_ = 0; s_ < NW; ++s_)                                            \
      _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_)                                           \
        wr[slot][s_][i_] = LS_STREAM_LOAD(reinterpret_cast<const u32x4*>(W + woff[s_][i_] + kb_)); \
  }
#define LS_LOAD_X(slot, blk)                                                                     \
  {                                                                                              \
    const size_t kb_ = (size_t)(blk) << 7;                                                       \
    _Pragma("unroll") for (int t_ = 0; t_ < MT; ++t_)                                            \
      _Pragma("unroll") for (int k_ = 0; k_ < 4; ++k_)                                           \
        xr[slot][t_][k_] = *reinterpret_cast<const u32x4*>(X + xoff[t_] + kb_ + k_ * 32);        \
  }
#define LS_LOAD_BLOCK(slot, blk) { LS_LOAD_W(slot, blk) LS_LOAD_X(slot, blk) }
  // the first weight block is requested before any other address is worked out: the sooner
  // the stream starts, the shorter the kernel (every wavefront has at least one block)
  LS_LOAD_W(0, b0)
  __builtin_amdgcn_sched_barrier(0);

  size_t xoff[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) xoff[t] = (size_t)min(lr + 16 * t, M - 1) * K + (size_t)(lg << 3);
  int a_off[4];  // LDS byte offset of the A fragment of k-step kk
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) a_off[kk] = lr * 256 + (((kk * 4 + lg) ^ lr) << 4);

  u32x4 xr[PF][MT][4];
  f32x4 acc[NW][MT];
#pragma unroll
  for (int s = 0; s < NW; ++s)
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[s][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // NORM (<= 16 rows): wave w owns rows 4w..4w+3 of the 1/rms computation.  It requests their
  // partial sums of squares straight into LDS (no registers held) BEFORE its activation loads, 16
  // bytes per lane, so one request covers 256 partials of a row (K is a multiple of 128, so a
  // row of K/16 partials is a whole number of 16-byte pieces).  Loads complete in order: once
  // the first block (weights and activations) has arrived the partials are there too, and the wave turns them
  // into 1/rms while the stream is in flight.
  typedef __attribute__((address_space(3))) void lds_void;
  const int pchunks = (fu.n_part + 255) >> 8;                         // 256-partial requests per row
  float* ss_lds = reinterpret_cast<float*>(smem + KS * (NW * 4096));  // [M][pchunks * 256]
  if constexpr (NORM && MT == 1) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = wave * 4 + r;
      for (int ch = 0; ch < pchunks; ++ch) {
        const int idx = ch * 256 + lane * 4;
        if (row < M && idx < fu.n_part)
          __builtin_amdgcn_global_load_lds((const void*)(fu.ss_in + (size_t)row * fu.n_part + idx),
                                           (lds_void*)(ss_lds + (row * pchunks + ch) * 256), 16, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  LS_LOAD_X(0, b0)
#pragma unroll
  for (int p = 1; p < PF; ++p)
    if (p < nb) LS_LOAD_BLOCK(p, b0 + p)

  // residual epilogue: the element this thread will update is known now; fetch it while the
  // weights stream so that its latency is not added after the K-split reduction
  float resid_pre = 0.f, gain_pre = 1.f;  // gain_pre: the gain of this thread's column
  if constexpr (EPI == EPI_RESID) {
    const int e0 = threadIdx.x;
    if (e0 < MT * 256 && (e0 >> 8) * 16 + ((e0 >> 4) & 15) < M)
      resid_pre = resid[(size_t)((e0 >> 8) * 16 + ((e0 >> 4) & 15)) * N + n0 + (e0 & 15)];
    if (fu.gamma_out) gain_pre = (float)fu.gamma_out[n0 + (threadIdx.x & 15)];
  }

  for (int b = 0; b < nb; b += PF) {
#pragma unroll
    for (int sl = 0; sl < PF; ++sl) {
      if (b + sl < nb) {
        // registers -> wave-private LDS scratch (lane-linear: conflict free)
#pragma unroll
        for (int s = 0; s < NW; ++s)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            *reinterpret_cast<u32x4*>(scratch + s * 4096 + i * 1024 + lane * 16) = wr[sl][s][i];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
          for (int s = 0; s < NW; ++s) {
            const bf16x8 af = *reinterpret_cast<const bf16x8*>(scratch + s * 4096 + a_off[kk]);
#pragma unroll
            for (int t = 0; t < MT; ++t) {
              const bf16x8 xf = __builtin_bit_cast(bf16x8, xr[sl][t][kk]);
              acc[s][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, xf, acc[s][t], 0, 0, 0);
            }
          }
        }
        // refill this ring slot with the block PF ahead
        if (b + sl + PF < nb) LS_LOAD_BLOCK(sl, b0 + b + sl + PF)
        if constexpr (NORM && MT == 1) {
          if (sl == 0 && b == 0) {
            __builtin_amdgcn_sched_barrier(0);  // stay behind the wait for the first weight block
            // the first weight block has arrived, hence this wave's partial sums too: 16 lanes
            // share a row, a lane adds every 16th partial in index order, then the fixed exchange
            const int row = wave * 4 + (lane >> 4);
            float ss = 0.f;
            if (row < M)
              for (int idx = lane & 15; idx < fu.n_part; idx += 16) ss += ss_lds[row * (pchunks * 256) + idx];
            ss = row16_sum(ss);
            if (row < M && (lane & 15) == 0) sm_inv[row] = 1.0f / sqrtf(ss / (float)K + fu.eps);
          }
        }
      }
    }
  }
#undef LS_LOAD_BLOCK
#undef LS_LOAD_W
#undef LS_LOAD_X

  // ---- sum the KS partial tiles in wave order (through an LDS area of their own: no wait for
  // the other waves' scratch to fall idle), then the epilogue
  if constexpr (NORM && MT > 1) {
    // more than 16 rows: 1/rms per row straight from the partial sums in global memory
    for (int row = threadIdx.x >> 4; row < M; row += KS * 4) {
      float ss = 0.f;
      for (int idx = threadIdx.x & 15; idx < fu.n_part; idx += 16) ss += fu.ss_in[(size_t)row * fu.n_part + idx];
      ss = row16_sum(ss);
      if ((threadIdx.x & 15) == 0) sm_inv[row] = 1.0f / sqrtf(ss / (float)K + fu.eps);
    }
  }
  float* red = reinterpret_cast<float*>(smem + KS * (NW * 4096) +
                                       ((NORM && MT == 1) ? M * pchunks * 1024 : 0));  // [KS][NW][MT][16 m][16 n]
#pragma unroll
  for (int s = 0; s < NW; ++s)
#pragma unroll
    for (int t = 0; t < MT; ++t)
      *reinterpret_cast<f32x4*>(red + ((((wave * NW + s) * MT + t) * 16 + lr) * 16 + lg * 4)) = acc[s][t];
  __syncthreads();
  for (int e = threadIdx.x; e < MT * 256; e += KS * 64) {
    const int t = e >> 8, ml = (e >> 4) & 15, n = e & 15;
    const int m = t * 16 + ml;
    if (m >= M) continue;  // whole 16-lane groups leave together
    float v[NW];
#pragma unroll
    for (int s = 0; s < NW; ++s) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < KS; ++w) sum += red[(((w * NW + s) * MT + t) * 16 + ml) * 16 + n];
      if constexpr (NORM) sum *= sm_inv[m];
      v[s] = sum;
    }
    const size_t o = (size_t)m * N + n0 + n;
    if constexpr (EPI == EPI_STORE) ((bf16*)outv)[o] = (bf16)v[0];
    else if constexpr (EPI == EPI_RESID) {
      const float xn = (e == (int)threadIdx.x ? resid_pre : resid[o]) + v[0];
      resid[o] = xn;
      if (fu.xb_out) {
        fu.xb_out[o] = (bf16)(xn * gain_pre);  // n == threadIdx.x % 16 in every pass of this loop
        const float ss = row16_sum(xn * xn);  // over the 16 columns of this tile, fixed order
        if (n == 0) fu.ss_out[(size_t)m * (N >> 4) + blockIdx.x] = ss;
      }
    }
    else if constexpr (EPI == EPI_SWIGLU) ((bf16*)outv)[o] = (bf16)(silu_f(v[0]) * v[NW - 1]);
    else ((float*)outv)[o] = v[0];
  }
}

#ifndef LS_SKINNY_PF
#define LS_SKINNY_PF 0
#endif
template <int MT, int EPI, int KS, bool NORM>
void launch_kn(const void* X, const void* W, int M, int N, int K, void* out, float* resid, const SkinnyFusion& fu,
               hipStream_t st) {
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  // register ring depth in 128-wide K blocks; two blocks measured best for every shape (a
  // deeper ring costs registers, hence resident wavefronts; also with one 8-wave workgroup
  // per CU, where registers are free, rings of 3 and 4 blocks and 16 waves ran 0.5-1.6% slower
  // per decode step: these short kernels are bound by their start and end, not by bytes in flight)
  constexpr int PF = LS_SKINNY_PF ? LS_SKINNY_PF : 2;
  // behind the waves' scratch areas: the rows' partial sums of squares (NORM kernel for <= 16
  // rows), then the K-split partial tiles
  const int scratch = KS * NW * 4096;
  const int ss_bytes = (NORM && MT == 1) ? M * ((fu.n_part + 255) / 256) * 1024 : 0;
  const int smem = scratch + ss_bytes + KS * NW * MT * 1024;
  static std::atomic<int> lds_allowed[64];
  allow_dynamic_lds_up_to((const void*)k_gemm_skinny<MT, EPI, KS, PF, NORM>, smem, lds_allowed);
  launch_kernel(k_gemm_skinny<MT, EPI, KS, PF, NORM>, dim3(N / 16), dim3(KS * 64), smem, st, (const bf16*)X,
                (const bf16*)W, M, N, K, out, resid, fu);
}

template <int MT, int EPI, int KS>
void launch_k(const void* X, const void* W, int M, int N, int K, void* out, float* resid, const SkinnyFusion& fu,
              hipStream_t st) {
  if constexpr (EPI == EPI_STORE || EPI == EPI_SWIGLU) {
    if (fu.ss_in) { launch_kn<MT, EPI, KS, true>(X, W, M, N, K, out, resid, fu, st); return; }
  }
  launch_kn<MT, EPI, KS, false>(X, W, M, N, K, out, resid, fu, st);
}

template <int MT, int EPI>
void launch_ks(const void* X, const void* W, int M, int N, int K, void* out, float* resid, int ks,
               const SkinnyFusion& fu, hipStream_t st) {
  if (ks == 0) {
    // measured with cold weights: 4 waves per workgroup stream best once there are >= 512
    // workgroups; with fewer (N = 4096: 256 of them) 8 waves keep more bytes in flight per CU
    ks = (N / 16) >= 512 ? 4 : 8;
    if (K / 128 < ks) ks = 4;
  }
  // 1024-thread workgroups leave too few registers for wide M or for two weight streams
  if (ks == 16 && (MT > 1 || EPI == EPI_SWIGLU)) ks = 8;
  if (ks == 8 && MT == 4 && EPI == EPI_SWIGLU) ks = 4;
  if (ks == 4) launch_k<MT, EPI, 4>(X, W, M, N, K, out, resid, fu, st);
  else if (ks == 8) launch_k<MT, EPI, 8>(X, W, M, N, K, out, resid, fu, st);
  else if constexpr (MT == 1) launch_k<MT, EPI, 16>(X, W, M, N, K, out, resid, fu, st);
}

template <int EPI>
void launch_mt(const void* X, const void* W, int M, int N, int K, void* out, float* resid, int ks,
               const SkinnyFusion& fu, hipStream_t st) {
  if (M <= 16) launch_ks<1, EPI>(X, W, M, N, K, out, resid, ks, fu, st);
  else if (M <= 32) launch_ks<2, EPI>(X, W, M, N, K, out, resid, ks, fu, st);
  else launch_ks<4, EPI>(X, W, M, N, K, out, resid, ks, fu, st);
}

}  // namespace

bool gemm_skinny_supported(int M, int N, int K) {
  return M >= 1 && M <= 64 && N >= 16 && N % 16 == 0 && K >= 512 && K % 128 == 0;
}

void launch_gemm_skinny(Epilogue epi, const void* X, const void* W, int M, int N, int K, void* out, float* resid,
                        int ks, hipStream_t st, const SkinnyFusion* fusion) {
  const SkinnyFusion fu = fusion ? *fusion : SkinnyFusion{};
  switch (epi) {
    case EPI_STORE: launch_mt<EPI_STORE>(X, W, M, N, K, out, resid, ks, fu, st); break;
    case EPI_RESID: launch_mt<EPI_RESID>(X, W, M, N, K, out, resid, ks, fu, st); break;
    case EPI_SWIGLU: launch_mt<EPI_SWIGLU>(X, W, M, N, K, out, resid, ks, fu, st); break;
    case EPI_F32: launch_mt<EPI_F32>(X, W, M, N, K, out, resid, ks, fu, st); break;
  }
}

}  // namespace ls
