// bf16 MFMA GEMM for the prompt pass: C[M,N] = A[M,K] W[N,K]^T, fp32 accumulation.
//
// One 512-thread workgroup (8 wavefronts, 2 x 4) owns a 256 x 256 tile of C and walks K in
// steps of 64.  Both operands are K-contiguous, so a lane's 16-byte global load is exactly
// the 8-element K slice an MFMA operand wants.  Tiles go from global memory straight into
// LDS (global_load_lds_dwordx4: no staging registers, no LDS store instructions) through a
// ring of NS stages: two stages of 64 KB by default.  One such instruction fills 1 KB = 8
// tile rows of 128 bytes; 16-byte chunks are XOR-swizzled by (row/2)&7 -- the lane that
// fills physical chunk p of row r fetches logical chunk p ^ ((r/2)&7) -- so that the 16 rows
// a quarter-wave reads for an MFMA operand fall into different banks (LDS has 64 banks
// here).  v_mfma_f32_32x32x16_bf16: the activation tile is the A operand (rows m), the
// weight tile the B operand (columns n); in the result a lane holds column n = lane%32 and
// rows 8*(r/4) + 4*(lane/32) + r%4, r = 0..15.
//
// K-step width and ring depth are compile-time (LS_GEMM_BK 64 or 32, LS_GEMM_NS stages).
// Measured inside the stage: rings of 3, 4 and 5 stages of 32-wide K steps all run 6% slower
// than two stages of 64.  The depth of the ring does not matter; the rate at which one CU
// pulls lines out of L2 does (its vector cache sits stalled on outstanding requests for 44%
// of the kernel's cycles, L2 hit rate 79%), and 64-byte row pieces cost twice the requests
// of whole 128-byte lines.
//
// Workgroup ids are remapped so that the 32 workgroups resident on one XCD (ids congruent
// modulo 8 land on the same XCD) work on a 4 x 8 patch of neighbouring tiles and share
// their operand tiles through that XCD's L2.
#include "kernels.hpp"
#include "device_util.hpp"

namespace ls {

namespace {

#ifndef LS_GEMM_BK
#define LS_GEMM_BK 64
#endif
#ifndef LS_GEMM_NS
#define LS_GEMM_NS 2
#endif
#ifndef LS_GEMM_WAVES
#define LS_GEMM_WAVES 8
#endif
constexpr int BM = 256, BN = 256, BK = LS_GEMM_BK;
constexpr int NWAVE = LS_GEMM_WAVES;            // wavefronts per workgroup: 8 (2 x 4) or 4 (2 x 2)
constexpr int WCOLS = NWAVE / 2;                // wavefronts side by side along N
constexpr int TJ = BN / (WCOLS * 32);           // 32-column MFMA tiles per wavefront: 2 or 4
constexpr int NS = LS_GEMM_NS;                  // ring of NS stages, NS-1 fills in flight
constexpr int ROWB = BK * 2;                    // bytes per tile row
constexpr int CH = ROWB / 16;                   // 16-byte chunks per row
constexpr int RPI = 1024 / ROWB;                // rows per fill instruction
constexpr int FROWS = BM / NWAVE;               // tile rows of each operand that one wavefront fills
constexpr int FI = FROWS / RPI;                 // fill instructions per operand per wave
constexpr int KK = BK / 16;                     // MFMA k-steps per stage
constexpr int SH = (BK == 64) ? 1 : 2;          // swizzle: rows that share a bank group
constexpr int TILE_BYTES = BM * ROWB;           // per operand tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES;
constexpr int SMEM_BYTES = NS * STAGE_BYTES;
constexpr int GROUP_M = 4;
// s_waitcnt vmcnt(n), other counters untouched: all fills but those of the last NS-2 stages
constexpr int VM_KEEP = 2 * FI * (NS - 2);
constexpr int WAIT_KEEP = 0x0F70 | (VM_KEEP & 15) | ((VM_KEEP >> 4) << 14);

__device__ __forceinline__ int swz(int row, int chunk) {
  return row * ROWB + ((chunk ^ ((row >> SH) & (CH - 1))) << 4);
}

template <int EPI>
__global__ void __launch_bounds__(NWAVE * 64, 1)
k_gemm_mfma(const bf16* __restrict__ A, const bf16* __restrict__ W, int M, int N, int K,
            void* __restrict__ outv, float* __restrict__ resid, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr bool GLU = (EPI == EPI_SWIGLU);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WCOLS, wn = wave % WCOLS;

  // ---- workgroup id -> tile
  const int nt = tiles_m * tiles_n;
#ifndef LS_GEMM_MAP
#define LS_GEMM_MAP 0
#endif
#if LS_GEMM_MAP == 0
  const int per_xcd = (nt + 7) >> 3;
  const int l = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
#else
  // chunks of 32 consecutive tiles go round-robin over the 8 XCDs
  const int slot = blockIdx.x >> 3;
  const int l = ((slot >> 5) << 8) + ((blockIdx.x & 7) << 5) + (slot & 31);
#endif
  if (l >= nt) return;
#if LS_GEMM_MAP < 2
  const int in_group = GROUP_M * tiles_n;
  const int first_m = (l / in_group) * GROUP_M;
  const int gsz = min(tiles_m - first_m, GROUP_M);
  const int tm = first_m + (l % in_group) % gsz;
  const int tn = (l % in_group) / gsz;
#else
  // two-level order: groups of 16 tile rows; inside a group, columns of 8 tiles; inside a
  // column, patches of 4 rows, row index fastest.  32 consecutive tiles are a 4 x 8 patch, 256
  // consecutive tiles a 16 x 16 block of the output (ragged edges shrink the pieces).
  const int sg_tiles = 16 * tiles_n;
  const int g = min(l / sg_tiles, (tiles_m - 1) >> 4);
  const int R = min(16, tiles_m - 16 * g);
  const int li = l - g * sg_tiles;
  const int c = min(li / (R * 8), (tiles_n - 1) >> 3);
  const int w = min(8, tiles_n - 8 * c);
  const int lj = li - c * R * 8;
  const int pm = min(lj / (4 * w), (R - 1) >> 2);
  const int rr = min(4, R - 4 * pm);
  const int lk = lj - pm * 4 * w;
  const int tm = 16 * g + 4 * pm + lk % rr;
  const int tn = 8 * c + lk / rr;
#endif
  const int m0 = tm * BM;
  const int n0 = GLU ? tn * (BN / 2) : tn * BN;  // GLU: 128 output columns per tile

  // ---- global -> LDS: wave w fills tile rows 32w..32w+31 of both operands, 8 rows per
  // instruction; lane l supplies row 32w + 8i + l/8, physical chunk l%8
  const bf16* ap[FI];
  const bf16* wp[FI];
#pragma unroll
  for (int i = 0; i < FI; ++i) {
    const int row = wave * FROWS + i * RPI + lane / CH;
    const int c = (lane % CH) ^ ((row >> SH) & (CH - 1));
    const int am = min(m0 + row, M - 1);
    ap[i] = A + (size_t)am * K + c * 8;
    int wrow;
    if constexpr (GLU) {
      // tile row -> weight row: 32-row blocks alternate gate / up, so that a wave's two
      // column tiles are the gate and the up projection of the same 32 output columns
      const int blk = row >> 5;
      const int f = min(n0 + (blk >> 1) * 32 + (row & 31), N - 1);
      wrow = (blk & 1) * N + f;
    } else {
      wrow = min(n0 + row, N - 1);
    }
    wp[i] = W + (size_t)wrow * K + c * 8;
  }
  f32x16 acc[4][TJ];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int lr = lane & 31, lh = lane >> 5;
  const int KT = K / BK;
  // LDS byte offsets of this lane's operand reads
  int a_off[KK][4], b_off[KK][TJ];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
    for (int i = 0; i < 4; ++i) a_off[kk][i] = swz(wm * 128 + i * 32 + lr, kk * 2 + lh);
#pragma unroll
    for (int j = 0; j < TJ; ++j) b_off[kk][j] = TILE_BYTES + swz(wn * (TJ * 32) + j * 32 + lr, kk * 2 + lh);
  }
  typedef __attribute__((address_space(3))) void lds_void;
  const int fill_off = (wave * FROWS) * ROWB;  // this wave's first row inside an operand tile

#define LS_FILL_TILE(buf, k0)                                                                          \
  _Pragma("unroll") for (int i = 0; i < FI; ++i) {                                                     \
    __builtin_amdgcn_global_load_lds((const void*)(ap[i] + (k0)),                                      \
        (lds_void*)(smem + (buf) * STAGE_BYTES + fill_off + i * 1024), 16, 0, 0);                      \
    __builtin_amdgcn_global_load_lds((const void*)(wp[i] + (k0)),                                      \
        (lds_void*)(smem + (buf) * STAGE_BYTES + TILE_BYTES + fill_off + i * 1024), 16, 0, 0);         \
  }
  // operand fragments are double buffered in registers: the LDS reads of k-step kk+1 are
  // issued before the MFMAs of k-step kk, so the matrix pipe does not wait on LDS latency
#define LS_READ_FRAGS(buf, kk, set)                                                                \
  {                                                                                                \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                  \
      af[set][i] = *reinterpret_cast<const bf16x8*>(smem + (buf) * STAGE_BYTES + a_off[kk][i]); \
    _Pragma("unroll") for (int j = 0; j < TJ; ++j)                                                 \
      bfr[set][j] = *reinterpret_cast<const bf16x8*>(smem + (buf) * STAGE_BYTES + b_off[kk][j]); \
  }
#define LS_MFMA_STEP(set)                                                                          \
  _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                    \
    _Pragma("unroll") for (int j = 0; j < TJ; ++j)                                                 \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][i], bfr[set][j], acc[i][j], 0, 0, 0);
  // within a k-step the six fragment reads of the next k-step are spread between the eight
  // MFMAs (one read after each of the first six) instead of being issued as one burst
#define LS_INTERLEAVE()                                                         \
  _Pragma("unroll") for (int g_ = 0; g_ < 4 + TJ; ++g_) {                       \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); /* one MFMA */           \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); /* one LDS read */       \
  }                                                                             \
  __builtin_amdgcn_sched_group_barrier(0x008, 4 * TJ - (4 + TJ), 0);
#define LS_COMPUTE_TILE(buf)                                    \
  {                                                             \
    bf16x8 af[2][4], bfr[2][TJ];                                \
    LS_READ_FRAGS(buf, 0, 0)                                    \
    __builtin_amdgcn_sched_barrier(0);                          \
    _Pragma("unroll") for (int kk = 0; kk < KK; ++kk) {         \
      if (kk + 1 < KK) LS_READ_FRAGS(buf, kk + 1, (kk + 1) & 1) \
      LS_MFMA_STEP(kk & 1)                                      \
      if (kk + 1 < KK) {                                        \
        LS_INTERLEAVE()                                         \
        __builtin_amdgcn_sched_barrier(0);                      \
      }                                                         \
    }                                                           \
  }
  // the barrier between k-steps: this wave's LDS reads are done (lgkmcnt) and the fills it
  // issued for the next stage have landed (vmcnt; younger fills stay in flight)
#define LS_STEP_BARRIER(imm)                 \
  asm volatile("" ::: "memory");             \
  __builtin_amdgcn_s_waitcnt(imm);           \
  __builtin_amdgcn_s_waitcnt(0xC07F);        \
  __builtin_amdgcn_sched_barrier(0);         \
  __builtin_amdgcn_s_barrier();              \
  __builtin_amdgcn_sched_barrier(0);         \
  asm volatile("" ::: "memory");

#ifndef LS_GEMM_ROT
#define LS_GEMM_ROT 1
#endif
#if LS_GEMM_ROT
  // The loop is rotated by one MFMA group: the barrier that hands over the next stage sits
  // BEFORE the last group of a k-step, so that group's MFMAs run while the first operand
  // fragments of the next stage are on their way from LDS, and neither wavefront of a SIMD
  // starts a k-step by waiting for LDS.  Right after the barrier the stage just read out is
  // refilled, which leaves its fills a whole k-step to land, as before.
  static_assert(NS == 2 && KK % 2 == 0, "the rotated loop alternates two stages and two fragment sets");
  {
    bf16x8 af[2][4], bfr[2][TJ];
    LS_FILL_TILE(0, 0)
    LS_STEP_BARRIER(0x0F70)
    if (KT > 1) LS_FILL_TILE(1, BK)
    LS_READ_FRAGS(0, 0, 0)
    __builtin_amdgcn_sched_barrier(0);
    for (int kt = 0; kt + 1 < KT; ++kt) {
      const int buf = kt & 1;
#pragma unroll
      for (int kk = 0; kk + 1 < KK; ++kk) {
        LS_READ_FRAGS(buf, kk + 1, (kk + 1) & 1)
        LS_MFMA_STEP(kk & 1)
        LS_INTERLEAVE()
        __builtin_amdgcn_sched_barrier(0);
      }
      // stage kt+1 has landed for every wavefront, and every wavefront has read all of stage kt
      LS_STEP_BARRIER(0x0F70)
      if (kt + 2 < KT) LS_FILL_TILE(buf, (kt + 2) * BK)
      LS_READ_FRAGS(buf ^ 1, 0, 0)
      LS_MFMA_STEP(1)
      LS_INTERLEAVE()
      __builtin_amdgcn_sched_barrier(0);
    }
    {  // the last k-step has nothing to hand over
      const int buf = (KT - 1) & 1;
#pragma unroll
      for (int kk = 0; kk + 1 < KK; ++kk) {
        LS_READ_FRAGS(buf, kk + 1, (kk + 1) & 1)
        LS_MFMA_STEP(kk & 1)
        LS_INTERLEAVE()
        __builtin_amdgcn_sched_barrier(0);
      }
      LS_MFMA_STEP(1)
    }
  }
#else
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < KT) LS_FILL_TILE(s, s * BK)
  if (KT >= NS - 1) { LS_STEP_BARRIER(WAIT_KEEP) } else { LS_STEP_BARRIER(0x0F70) }
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt % NS;
    // stage (kt-1) % NS was last read in step kt-1, which every wave has left (barrier)
    const bool more = kt + NS - 1 < KT;
    if (more) LS_FILL_TILE((kt + NS - 1) % NS, (kt + NS - 1) * BK)
    LS_COMPUTE_TILE(buf)
    if (more) { LS_STEP_BARRIER(WAIT_KEEP) } else { LS_STEP_BARRIER(0x0F70) }
  }
#endif
#undef LS_FILL_TILE
#undef LS_COMPUTE_TILE
#undef LS_INTERLEAVE
#undef LS_READ_FRAGS
#undef LS_MFMA_STEP
#undef LS_STEP_BARRIER

  // ---- epilogue
  if constexpr (EPI == EPI_RESID) {
    // fp32 read-modify-write of the residual rows.  A store to `resid` may alias a later load
    // as far as the compiler can tell, so "resid[o] += acc" element by element would wait one
    // memory round trip per element; here the 16 old values of the NEXT 32 x 32 tile are
    // requested before the current tile's sums are stored, so every lane always has 16 loads in
    // flight behind its stores.
    float old[2][16];
    const int ncol = n0 + wn * (TJ * 32) + lr;
#define LS_RESID_LOAD(t, set)                                                                       \
  _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                  \
    const int m_ = m0 + wm * 128 + ((t) / TJ) * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);               \
    const int n_ = ncol + ((t) % TJ) * 32;                                                          \
    old[set][r] = (m_ < M && n_ < N) ? resid[(size_t)m_ * N + n_] : 0.f;                            \
  }
    LS_RESID_LOAD(0, 0)
#pragma unroll
    for (int t = 0; t < 4 * TJ; ++t) {
      if (t + 1 < 4 * TJ) LS_RESID_LOAD(t + 1, (t + 1) & 1)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 128 + (t / TJ) * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
        const int n = ncol + (t % TJ) * 32;
        if (m < M && n < N) resid[(size_t)m * N + n] = old[t & 1][r] + acc[t / TJ][t % TJ][r];
      }
    }
#undef LS_RESID_LOAD
    return;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
      if (m >= M) continue;
      if constexpr (GLU) {
#pragma unroll
        for (int jj = 0; jj < TJ / 2; ++jj) {
          const int n = n0 + wn * (TJ * 16) + jj * 32 + lr;
          if (n < N) ((bf16*)outv)[(size_t)m * N + n] = (bf16)(silu_f(acc[i][2 * jj][r]) * acc[i][2 * jj + 1][r]);
        }
      } else {
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
          const int n = n0 + wn * (TJ * 32) + j * 32 + lr;
          if (n >= N) continue;
          const size_t o = (size_t)m * N + n;
          if constexpr (EPI == EPI_STORE) ((bf16*)outv)[o] = (bf16)acc[i][j][r];
          else ((float*)outv)[o] = acc[i][j][r];
        }
      }
    }
  }
}

template <int EPI>
void launch_t(const void* A, const void* W, int M, int N, int K, void* out, float* resid, hipStream_t st) {
  static std::atomic<uint64_t> lds_allowed{0};
  allow_dynamic_lds((const void*)k_gemm_mfma<EPI>, SMEM_BYTES, lds_allowed);
  const int tiles_m = (M + BM - 1) / BM;
  const int ncols = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  const int tiles_n = (N + ncols - 1) / ncols;
  const int nt = tiles_m * tiles_n;
#if LS_GEMM_MAP == 0
  const int grid = ((nt + 7) / 8) * 8;
#else
  const int grid = ((nt + 255) / 256) * 256;
#endif
  launch_kernel(k_gemm_mfma<EPI>, dim3(grid), dim3(NWAVE * 64), SMEM_BYTES, st, (const bf16*)A, (const bf16*)W, M, N, K, out,
                resid, tiles_m, tiles_n);
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
