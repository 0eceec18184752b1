// bf16 MFMA GEMM for the prompt pass: C[M,N] = A[M,K] W[N,K]^T, fp32 accumulation.
//
// One 512-thread workgroup (8 wavefronts, 2 x 4) owns a 256 x 256 tile of C and walks K in
// steps of 64.  Both operands are K-contiguous, so a lane's 16-byte global load is exactly
// the 8-element K slice an MFMA operand wants.  Tiles are staged in LDS (double buffered,
// 128 KB), 16-byte chunks XOR-swizzled by row so that the 32 rows an MFMA operand read
// touches fall into different banks.  v_mfma_f32_32x32x16_bf16: the activation tile is the
// A operand (rows m), the weight tile the B operand (columns n); in the result a lane holds
// column n = lane%32 and rows 8*(r/4) + 4*(lane/32) + r%4, r = 0..15.
//
// Workgroup ids are remapped so that the 32 workgroups resident on one XCD (ids congruent
// modulo 8 land on the same XCD) work on a 4 x 8 patch of neighbouring tiles and share
// their operand tiles through that XCD's L2.
#include "kernels.hpp"
#include "device_util.hpp"

namespace ls {

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = BM * BK * 2;         // 32 KB per operand tile
constexpr int SMEM_BYTES = 4 * TILE_BYTES;      // A and W, two buffers each
constexpr int GROUP_M = 4;

#ifndef LS_GEMM_SWZ_SHIFT
#define LS_GEMM_SWZ_SHIFT 1
#endif
__device__ __forceinline__ int swz(int row, int chunk) {
  return row * 128 + ((chunk ^ ((row >> LS_GEMM_SWZ_SHIFT) & 7)) << 4);
}

template <int EPI>
__global__ void __launch_bounds__(512, 1)
k_gemm_mfma(const bf16* __restrict__ A, const bf16* __restrict__ W, int M, int N, int K,
            void* __restrict__ outv, float* __restrict__ resid, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr bool GLU = (EPI == EPI_SWIGLU);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  // ---- workgroup id -> tile, XCD-aware and grouped along M
  const int nt = tiles_m * tiles_n;
  const int per_xcd = (nt + 7) >> 3;
  const int l = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (l >= nt) return;
  const int in_group = GROUP_M * tiles_n;
  const int first_m = (l / in_group) * GROUP_M;
  const int gsz = min(tiles_m - first_m, GROUP_M);
  const int tm = first_m + (l % in_group) % gsz;
  const int tn = (l % in_group) / gsz;
  const int m0 = tm * BM;
  const int n0 = GLU ? tn * (BN / 2) : tn * BN;  // GLU: 128 output columns per tile

  // ---- global -> register staging: thread owns chunk c of rows r0 + 64 i
  const int c = tid & 7, r0 = tid >> 3;
  const bf16* ap[4];
  const bf16* wp[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int row = r0 + 64 * i;
    int am = min(m0 + row, M - 1);
    ap[i] = A + (size_t)am * K + c * 8;
    int wrow;
    if constexpr (GLU) {
      // tile row -> weight row: 32-row blocks alternate gate / up, so that a wave's two
      // column tiles are the gate and the up projection of the same 32 output columns
      int blk = row >> 5;
      int f = min(n0 + (blk >> 1) * 32 + (row & 31), N - 1);
      wrow = (blk & 1) * N + f;
    } else {
      wrow = min(n0 + row, N - 1);
    }
    wp[i] = W + (size_t)wrow * K + c * 8;
  }
  u32x4 ra[4], rw[4];
  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int lr = lane & 31, lh = lane >> 5;
  const int KT = K / BK;
  // LDS byte offsets of this thread's staging chunks and of its operand reads
  int st_off[4], a_off[4][4], b_off[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i) st_off[i] = swz(r0 + 64 * i, c);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
    for (int i = 0; i < 4; ++i) a_off[kk][i] = swz(wm * 128 + i * 32 + lr, kk * 2 + lh);
#pragma unroll
    for (int j = 0; j < 2; ++j) b_off[kk][j] = TILE_BYTES + swz(wn * 64 + j * 32 + lr, kk * 2 + lh);
  }

#define LS_LOAD_TILE(k0)                                              \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) {                     \
    ra[i] = *reinterpret_cast<const u32x4*>(ap[i] + (k0));            \
    rw[i] = *reinterpret_cast<const u32x4*>(wp[i] + (k0));            \
  }
#define LS_STORE_TILE(buf)                                                                   \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                            \
    *reinterpret_cast<u32x4*>(smem + (buf) * 2 * TILE_BYTES + st_off[i]) = ra[i];            \
    *reinterpret_cast<u32x4*>(smem + (buf) * 2 * TILE_BYTES + TILE_BYTES + st_off[i]) = rw[i]; \
  }
#define LS_COMPUTE_TILE(buf)                                                                     \
  _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                             \
    bf16x8 af[4], bfr[2];                                                                        \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                \
      af[i] = *reinterpret_cast<const bf16x8*>(smem + (buf) * 2 * TILE_BYTES + a_off[kk][i]);    \
    _Pragma("unroll") for (int j = 0; j < 2; ++j)                                                \
      bfr[j] = *reinterpret_cast<const bf16x8*>(smem + (buf) * 2 * TILE_BYTES + b_off[kk][j]);   \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                \
      _Pragma("unroll") for (int j = 0; j < 2; ++j)                                              \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);  \
  }

  LS_LOAD_TILE(0)
  LS_STORE_TILE(0)
  __syncthreads();
  for (int kt = 0; kt + 1 < KT; ++kt) {
    const int buf = kt & 1;
    LS_LOAD_TILE((kt + 1) * BK)
    LS_COMPUTE_TILE(buf)
    LS_STORE_TILE(buf ^ 1)
    __syncthreads();
  }
  {
    const int buf = (KT - 1) & 1;
    LS_COMPUTE_TILE(buf)
  }
#undef LS_LOAD_TILE
#undef LS_STORE_TILE
#undef LS_COMPUTE_TILE

  // ---- epilogue
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
      if (m >= M) continue;
      if constexpr (GLU) {
        const int n = n0 + wn * 32 + lr;
        if (n < N) ((bf16*)outv)[(size_t)m * N + n] = (bf16)(silu_f(acc[i][0][r]) * acc[i][1][r]);
      } else {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int n = n0 + wn * 64 + j * 32 + lr;
          if (n >= N) continue;
          const size_t o = (size_t)m * N + n;
          if constexpr (EPI == EPI_STORE) ((bf16*)outv)[o] = (bf16)acc[i][j][r];
          else if constexpr (EPI == EPI_RESID) resid[o] += acc[i][j][r];
          else ((float*)outv)[o] = acc[i][j][r];
        }
      }
    }
  }
}

template <int EPI>
void launch_t(const void* A, const void* W, int M, int N, int K, void* out, float* resid, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)k_gemm_mfma<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
    attr_set = true;
  }
  const int tiles_m = (M + BM - 1) / BM;
  const int ncols = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  const int tiles_n = (N + ncols - 1) / ncols;
  const int nt = tiles_m * tiles_n;
  const int grid = ((nt + 7) / 8) * 8;
  k_gemm_mfma<EPI><<<grid, 512, SMEM_BYTES, st>>>((const bf16*)A, (const bf16*)W, M, N, K, out, resid, tiles_m, tiles_n);
}

}  // namespace

bool gemm_mfma_supported(int M, int N, int K) { return M >= 1 && N >= 1 && K >= BK && K % BK == 0; }

void launch_gemm_mfma(Epilogue epi, const void* A, const void* W, int M, int N, int K, void* out, float* resid,
                      hipStream_t st) {
  switch (epi) {
    case EPI_STORE: launch_t<EPI_STORE>(A, W, M, N, K, out, resid, st); break;
    case EPI_RESID: launch_t<EPI_RESID>(A, W, M, N, K, out, resid, st); break;
    case EPI_SWIGLU: launch_t<EPI_SWIGLU>(A, W, M, N, K, out, resid, st); break;
    case EPI_F32: launch_t<EPI_F32>(A, W, M, N, K, out, resid, st); break;
  }
}

}  // namespace ls
