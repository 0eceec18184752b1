// bf16 MFMA GEMM for the prompt pass: C[M,N] = A[M,K] W[N,K]^T, fp32 accumulation, built on
// v_mfma_f32_16x16x32_bf16.
//
// Why this instruction: dense MFMA work on this chip is limited by power, not by issue slots.
// A register-only loop of v_mfma_f32_32x32x16_bf16 with varied operands settles at about
// 1.8 GHz (1.82 PFLOP/s), the same loop of v_mfma_f32_16x16x32_bf16 at 2.15 GHz
// (2.2 PFLOP/s), both at 2.4 GHz with all-zero operands: per multiply-add the 16x16x32 form
// moves half the fp32 accumulator bytes through the register file.
//
// Tile and data path: one 256-thread workgroup (4 wavefronts, 2 x 2, one per SIMD) owns a
// 256 x 256 tile of C and walks K in steps of 64.  Both operands are K-contiguous, so a lane's
// 16-byte global load is exactly the 8-element K slice an MFMA operand wants.  Tiles go from
// global memory straight into LDS (global_load_lds_dwordx4: no staging registers, no LDS store
// instructions) into a ring of two stages of 64 KB (LDS has no room for a third at this tile
// size, and rings of narrower k-steps measured slower: 64-byte row pieces cost twice the
// requests of whole 128-byte lines).  One such instruction fills 1 KB = 8 tile rows of 128
// bytes; 16-byte chunks are XOR-swizzled by (row/2)&7 -- the lane that fills physical chunk p
// of row r fetches logical chunk p ^ ((r/2)&7) -- so that the 16 rows a quarter-wave reads for
// an MFMA operand fall into different banks (LDS has 64 banks here).
//
// A wavefront owns 128 rows x 128 columns of C = 8 x 8 MFMA tiles of 16 x 16; the 256
// accumulator registers live in the AGPR half of a wavefront's 512 registers, the operand
// fragments of a half-step (8 + 8 of 4 registers) in two sets in the VGPR half.  The weight
// fragment is the instruction's A operand and the activation fragment its B operand, so in
// the result a lane holds row m = lane%16 of the tile and FOUR CONSECUTIVE columns
// n = 4*(lane/16) .. +3.
//
// Why four wavefronts of 128 x 128 and not eight of 128 x 64 (the previous version of this
// kernel, two per SIMD): shader-clock stamps around the hand-over showed that of the two
// wavefronts of a SIMD the older one is served first by the matrix pipe: it finished its 64
// MFMAs of a k-step (1024 cycles of matrix work) after 1480 cycles and then waited 1160 cycles
// at the barrier, while the younger one needed 2460 -- alone on the SIMD for the last third,
// where a single instruction stream with its own waits kept the pipe only two thirds busy.
// One wavefront per SIMD has nobody to wait for (all four arrive within 20 cycles of each
// other), reads a third fewer operand bytes from LDS per multiply-add, and its k-loop took
// 109.5 us per 256 x 256 x 5120 tile against 114.5; what it loses is the second wavefront that
// covered the issue slots of the memory instructions and half of the memory-level parallelism
// in the epilogues.  With one wavefront per SIMD every instruction between two MFMAs costs the
// matrix pipe its own issue time: a k-step's 128 MFMAs need 2048 cycles and take 2250 with the
// LDS reads alone (about 5 cycles per ds_read_b128), 2460 with the fills (about 12 per
// global_load_lds), 2740 with the hand-over.  (Measured without effect: four fills sharing one
// LDS base in M0 through the instruction's immediate offset, which removes twelve scalar
// writes and wait states per k-step; starting the eight XCDs a few microseconds apart so that
// their epilogues do not ask for HBM at the same time.)
//
// The k-loop is written out in issue order.  A k-step is two half-steps of 64 MFMAs (k = 32
// each).  The LDS reads are inline assembly and the waits for them are explicit
// s_waitcnt lgkmcnt(n) with the exact number of younger reads that may still be in flight:
// the compiler, which treats an LDS-direct load as a possible writer of anything in LDS, waits
// for ALL outstanding LDS reads before every dependent MFMA once such a load is in the
// function.  LDS reads return in order; the counts are derived next to the macros.
// The same compiler pass decides where the k-loop waits for vector memory: a register that it
// cannot prove free of a pending load when the loop is entered again after an epilogue (a
// spilled value reloaded on one path, a load whose result one branch does not use) makes it
// put s_waitcnt vmcnt(0) in front of an MFMA INSIDE the k-loop, which then waits for every
// fill as soon as it is issued (20 % of a launch, seen twice).  Hence the straight-line
// epilogues, the lane numbers that pass through empty asm statements (so that what is derived
// from them is computed where it is used and nothing is spilled across the loop), and the
// scheduling barriers between the row blocks of an epilogue.
//
// Stage hand-over: the barrier sits between the two half-steps of a k-step.  Before it a
// wavefront has issued and completed every read of the stage being retired (the second
// half-step's fragments were all requested during the first) and has seen its own fills of
// the next stage land; after it the second half-step computes from registers, requests the
// next stage's first fragments and issues the fills that refill the retired stage.
//
// Persistent workgroups: 256 workgroups, one per CU, each walking tiles l, l + 256, ...; a
// workgroup's k-steps form ONE stream across its tiles.  The fills of a tile's last two
// k-steps fetch the first two k-blocks of the workgroup's next tile, so the next tile's first
// hand-over finds its data there, and the epilogue's stores drain while the next tile
// computes.  Wall-clock stamps per tile (development build, 13B shapes) of a version that
// launched one workgroup per tile: 2.2-2.5 us from a workgroup's start to its first hand-over
// and 1.2 / 2.6 / 7.4 us (QKV / gate-up / residual GEMMs) between one workgroup's end and the
// next one's start on the same CU, against 114 us of k-loop per tile at K = 5120.  What remains
// outside the k-loop is the epilogue itself, with the matrix pipe idle: 4 us (SwiGLU), 10 us
// (RoPE and cache append), 18 us (fp32 residual read-modify-write) per tile.
//
// Fills that miss L2 cost wall time, so every workgroup touches its share of the operand
// lines one k-step ahead (see the L2 prefetch below).
//
// Tile order: the 32 workgroups resident on one XCD (ids congruent modulo 8 land on the same
// XCD) work on a 4 x 8 patch of neighbouring tiles and share their operand panels through that
// XCD's L2, and the eight XCDs work on the eight patches of one 16 x 16 block of tiles at the
// same time and find each other's panels in the memory-side cache (+1.2 % over patches that
// are far apart).
#include "kernels.hpp"
#include "device_util.hpp"

namespace ls {

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NWAVE = 4;
constexpr int ROWB = BK * 2;               // bytes per tile row
constexpr int TILE_BYTES = BM * ROWB;      // 32 KB per operand tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES;
constexpr int SMEM_BYTES = 2 * STAGE_BYTES;
constexpr int FI = 8;                      // fill instructions per operand per wavefront and stage
constexpr int PERSISTENT_WGS = 256;        // one workgroup per CU
constexpr int PF_AHEAD = 1;                // k-steps between the L2 prefetch of a line and its fill

__device__ __forceinline__ unsigned swz(int row, int chunk) {
  return (unsigned)(row * ROWB + ((chunk ^ ((row >> 1) & 7)) << 4));
}


// Tile number l in the two-level order -> tile coordinates, position inside its 4 x 8 patch
// (q4 of rr rows, q8 of w columns; ragged edges shrink the patch).
struct TileAt { int tm, tn, q4, q8; bool full; };
__device__ __forceinline__ TileAt tile_at(int l, int tiles_m, int tiles_n) {
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
  TileAt t;
  t.tm = 16 * g + 4 * pm + lk % rr;
  t.tn = 8 * c + lk / rr;
  t.q4 = lk % rr;
  t.q8 = lk / rr;
  t.full = rr == 4 && w == 8;  // a whole patch: its 32 workgroups run side by side on one XCD
  return t;
}

// Two result fragments that lie side by side (16 + 16 columns of the same 16 rows), as four
// bf16 values per lane each -> eight consecutive columns per lane: lane (row, q) ends up with
// columns 8q..8q+7 of the 32, so that the four lanes of a row store 64 contiguous bytes with
// one 16-byte store each instead of 4 x 8 bytes twice (a store instruction is sixteen row
// segments for the memory pipeline whatever their width: half the instructions, half the
// requests).  The data moves between the wavefront's four 16-lane rows with the two swap
// instructions of this chip: v_permlane32_swap exchanges rows 2,3 of its first operand with rows
// 0,1 of its second, v_permlane16_swap rows 1,3 of the first with rows 0,2 of the second.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 side_by_side(bf16x4 a, bf16x4 b) {
  const u32x2 ua = __builtin_bit_cast(u32x2, a), ub = __builtin_bit_cast(u32x2, b);
  u32x4 o;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    // rows after the first swap: first = a0 a1 b0 b1, second = a2 a3 b2 b3 (a2: a's value in row 2)
    const u32x2 s = __builtin_amdgcn_permlane32_swap(ua[h], ub[h], false, false);
    // after the second: first = a0 a2 b0 b2, second = a1 a3 b1 b3
    const u32x2 t = __builtin_amdgcn_permlane16_swap(s[0], s[1], false, false);
    o[h] = t[0];      // columns 8q + 2h, +1: from the fragment's row 2(q%2)
    o[2 + h] = t[1];  // columns 8q + 4 + 2h, +1: from row 2(q%2) + 1
  }
  return o;
}
// a where every bit of mask is set, b where none is (a select the compiler cannot turn into a branch)
__device__ __forceinline__ float pick_bits(unsigned mask, float a, float b) {
  return __uint_as_float((__float_as_uint(a) & mask) | (__float_as_uint(b) & ~mask));
}
__device__ __forceinline__ bf16x4 to_bf16x4(f32x4 v) {
  bf16x4 y;
#pragma unroll
  for (int r = 0; r < 4; ++r) y[r] = (bf16)v[r];
  return y;
}

constexpr int EPI_ROPE = 4;  // EPI_STORE with RoPE and the KV-cache append (QKV projection of a prompt pass)

// Epilogue of one tile, for one 64-column slice of a wavefront's 128 x 128 results: the four
// fragments accf[i][J0 .. J0 + 3], whose element r is
// C[m0 + 128 wm + 16 i + lane%16][n0 + 64 wn + 16 j + 4 (lane/16) + r] with wn the slice's
// number within the tile (0..3) and j = 0..3.
template <int EPI, int J0>
__device__ __forceinline__ void store_tile(f32x4 (&accf)[8][8], int m0, int n0, int M, int N, void* __restrict__ outv,
                                           float* __restrict__ resid, const RopeAppend& rp, int wm, int wn, int l16,
                                           int lq) {
#define acc(i_, j_) accf[i_][J0 + (j_)]
  // (opaque to the compiler, so that nothing derived from the lane number for this epilogue
  // is computed before the k-loop and kept in registers through it)
  asm volatile("" : "+v"(l16), "+v"(lq));
  constexpr bool GLU = (EPI == EPI_SWIGLU);
  const bool vec = (N & 3) == 0;
  if constexpr (EPI == EPI_ROPE) {
    // The slice's 64 columns lie inside one head (head_dim 64 or 128): query, key or value.
    // A lane's four consecutive columns are two rotation pairs (dims 2p, 2p+1); their
    // (cos, sin) are one 16-byte table load.  The table loads of the next row block are in
    // flight while the current one is rotated and stored.
    const int ncol0 = n0 + wn * 64;
    if (ncol0 >= N) return;  // N is a multiple of the head size: the whole slice is out
    const int head = ncol0 / rp.hd, dd0 = ncol0 - head * rp.hd;
    const bool is_q = head < rp.hq, is_v = head >= rp.hq + rp.hkv;
    const int kh = is_v ? head - rp.hq - rp.hkv : head - rp.hq;
    bf16* const cache = rp.kc + (is_v ? rp.vc - rp.kc : (ptrdiff_t)0);  // (a plain choice between the two pointers is compiled into a table in private memory)
    int pos[8], seq[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      // (no load here is conditional, and none is left unused on any path: a load that the
      // compiler cannot prove finished would make it wait for ALL vector memory operations,
      // fills included, inside the k-loop that follows this epilogue in the next tile)
      const int m = m0 + wm * 128 + i * 16 + l16, mm = min(m, M - 1);
      const int p = rp.row_pos[mm], sq = rp.row_seq[mm];
      pos[i] = m < M ? p : -1;
      seq[i] = sq;
    }
    // Straight-line code from here to the stores: table loads are made for value heads too and
    // the choice between a turned and an untouched value is a bit select, so that the compiler
    // has no branch to build around a load.
    f32x4 tab[2][4];
#define LS_TAB_LOAD(i_, set_)                                                                         \
  _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                       \
    tab[set_][j] = *reinterpret_cast<const f32x4*>(                                                   \
        rp.cs + ((size_t)max(pos[i_], 0) * (rp.hd >> 1) + ((dd0 + j * 16 + 4 * lq) >> 1)) * 2);
    LS_TAB_LOAD(0, 0)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_barrier(0);  // one row block at a time: the accumulators sit in AGPRs
      if (i + 1 < 8) { LS_TAB_LOAD(i + 1, (i + 1) & 1) }
      const int m = m0 + wm * 128 + i * 16 + l16;
      // a row past the end of the call stores nothing; a row whose sequence has no room left
      // keeps its query as projected and appends nothing, as with the separate rotation kernel
      const bool live = m < M && (pos[i] >= 0 || is_q);
      const unsigned turn = (!is_v && pos[i] >= 0) ? 0xFFFFFFFFu : 0u;
      bf16x4 y[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x4 v = acc(i, j);
        const f32x4 t = tab[i & 1][j];  // cos, sin of pair dd/2; cos, sin of pair dd/2 + 1
        // the projection's output is rounded to bf16 first, as the separate rotation kernel sees it
        const float u0 = (float)(bf16)v[0], u1 = (float)(bf16)v[1], u2 = (float)(bf16)v[2], u3 = (float)(bf16)v[3];
        f32x4 w;
        w[0] = pick_bits(turn, u0 * t[0] - u1 * t[1], v[0]);
        w[1] = pick_bits(turn, u0 * t[1] + u1 * t[0], v[1]);
        w[2] = pick_bits(turn, u2 * t[2] - u3 * t[3], v[2]);
        w[3] = pick_bits(turn, u2 * t[3] + u3 * t[2], v[3]);
        y[j] = to_bf16x4(w);
      }
      bf16* row = is_q ? (bf16*)outv + (size_t)m * N + ncol0
                       : cache + (((size_t)seq[i] * rp.hkv + kh) * rp.max_seq + max(pos[i], 0)) * rp.hd + dd0;
#pragma unroll
      for (int jp = 0; jp < 2; ++jp) {
        const u32x4 o = side_by_side(y[2 * jp], y[2 * jp + 1]);  // every lane takes part
        if (live) *reinterpret_cast<u32x4*>(row + jp * 32 + 8 * lq) = o;
      }
    }
#undef LS_TAB_LOAD
    return;
  }
  if constexpr (EPI == EPI_RESID) {
    // fp32 read-modify-write of the residual rows, 16 bytes per lane; the sixteen old values of
    // four row blocks are requested before the first sum is stored (the operand fragments'
    // registers are free by now)
    constexpr int RB = 4;
#pragma unroll
    for (int i2 = 0; i2 < 8; i2 += RB) {
      f32x4 old[RB][4];
#pragma unroll
      for (int ii = 0; ii < RB; ++ii)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int m = m0 + wm * 128 + (i2 + ii) * 16 + l16;
          const int n = n0 + wn * 64 + j * 16 + 4 * lq;
          const float* p = resid + (size_t)m * N + n;
          if (m < M && vec && n + 3 < N) old[ii][j] = *reinterpret_cast<const f32x4*>(p);
          else
#pragma unroll
            for (int r = 0; r < 4; ++r) old[ii][j][r] = (m < M && n + r < N) ? p[r] : 0.f;
        }
#pragma unroll
      for (int ii = 0; ii < RB; ++ii)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int m = m0 + wm * 128 + (i2 + ii) * 16 + l16;
          const int n = n0 + wn * 64 + j * 16 + 4 * lq;
          float* p = resid + (size_t)m * N + n;
          const f32x4 v = old[ii][j] + acc(i2 + ii, j);
          if (m < M && vec && n + 3 < N) *reinterpret_cast<f32x4*>(p) = v;
          else
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (m < M && n + r < N) p[r] = v[r];
        }
    }
    return;
  }
  if constexpr (EPI == EPI_STORE || GLU) {
    // bf16 results, the slice's columns all inside the matrix and rows 16-byte aligned:
    // 16-byte stores of eight consecutive columns (see side_by_side)
    constexpr int WCOLS = GLU ? 32 : 64;
    const int ncol0 = n0 + wn * WCOLS;
    if ((N & 7) == 0 && ncol0 + WCOLS <= N) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_barrier(0);  // one row block at a time: the accumulators sit in AGPRs
        const int m = m0 + wm * 128 + i * 16 + l16;
        bf16* row = (bf16*)outv + (size_t)min(m, M - 1) * N + ncol0 + 8 * lq;
        if constexpr (GLU) {
          f32x4 g[2];
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) g[j][r] = silu_f(acc(i, j)[r]) * acc(i, j + 2)[r];
          const u32x4 o = side_by_side(to_bf16x4(g[0]), to_bf16x4(g[1]));
          if (m < M) *reinterpret_cast<u32x4*>(row) = o;
        } else {
#pragma unroll
          for (int jp = 0; jp < 2; ++jp) {
            const u32x4 o = side_by_side(to_bf16x4(acc(i, 2 * jp)), to_bf16x4(acc(i, 2 * jp + 1)));
            if (m < M) *reinterpret_cast<u32x4*>(row + jp * 32) = o;
          }
        }
      }
      return;
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    __builtin_amdgcn_sched_barrier(0);  // one row block at a time: the accumulators sit in AGPRs
    const int m = m0 + wm * 128 + i * 16 + l16;
    if (m >= M) continue;
    if constexpr (GLU) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 32 + j * 16 + 4 * lq;
        bf16x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = (bf16)(silu_f(acc(i, j)[r]) * acc(i, j + 2)[r]);
        bf16* p = (bf16*)outv + (size_t)m * N + n;
        if (vec && n + 3 < N) *reinterpret_cast<bf16x4*>(p) = v;
        else
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (n + r < N) p[r] = v[r];
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int n = n0 + wn * 64 + j * 16 + 4 * lq;
        if constexpr (EPI == EPI_STORE) {
          bf16x4 v;
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = (bf16)acc(i, j)[r];
          bf16* p = (bf16*)outv + (size_t)m * N + n;
          if (vec && n + 3 < N) *reinterpret_cast<bf16x4*>(p) = v;
          else
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (n + r < N) p[r] = v[r];
        } else {
          float* p = (float*)outv + (size_t)m * N + n;
          if (vec && n + 3 < N) *reinterpret_cast<f32x4*>(p) = acc(i, j);
          else
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (n + r < N) p[r] = acc(i, j)[r];
        }
      }
    }
  }
#undef acc
}

// fp32 store of a wavefront's whole 128 x 128 results (the LM head's logits), 16 bytes per lane.
__device__ __forceinline__ void store_tile_f32(f32x4 (&acc)[8][8], int m0, int n0, int M, int N,
                                               float* __restrict__ out, int wm, int wn, int l16, int lq) {
  const bool vec = (N & 3) == 0;
  asm volatile("" : "+v"(l16), "+v"(lq));  // see store_tile
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    __builtin_amdgcn_sched_barrier(0);  // one row block at a time: the accumulators sit in AGPRs
    const int m = m0 + wm * 128 + i * 16 + l16;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int n = n0 + wn * 128 + j * 16 + 4 * lq;
      float* p = out + (size_t)min(m, M - 1) * N + n;
      const f32x4 v = acc[i][j];
      if (m < M && vec && n + 3 < N) *reinterpret_cast<f32x4*>(p) = v;
      else
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (m < M && n + r < N) p[r] = v[r];
    }
  }
}

// fp32 read-modify-write of the residual rows for a wavefront's whole 128 x 128 results, 16
// bytes per lane: the old values of RB row blocks (8 RB loads of 16 bytes per lane) are
// requested before the first sum is stored; the operand fragments' registers are free by then.
__device__ __forceinline__ void add_tile_to_residual(f32x4 (&acc)[8][8], int m0, int n0, int M, int N,
                                                     float* __restrict__ resid, int wm, int wn, int l16, int lq) {
  constexpr int RB = 4;
  const bool vec = (N & 3) == 0;
  asm volatile("" : "+v"(l16), "+v"(lq));  // see store_tile
#pragma unroll
  for (int i2 = 0; i2 < 8; i2 += RB) {
    __builtin_amdgcn_sched_barrier(0);
    f32x4 old[RB][8];
#pragma unroll
    for (int ii = 0; ii < RB; ++ii)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int m = m0 + wm * 128 + (i2 + ii) * 16 + l16;
        const int n = n0 + wn * 128 + j * 16 + 4 * lq;
        const float* p = resid + (size_t)m * N + n;
        if (m < M && vec && n + 3 < N) old[ii][j] = *reinterpret_cast<const f32x4*>(p);
        else
#pragma unroll
          for (int r = 0; r < 4; ++r) old[ii][j][r] = (m < M && n + r < N) ? p[r] : 0.f;
      }
#pragma unroll
    for (int ii = 0; ii < RB; ++ii)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int m = m0 + wm * 128 + (i2 + ii) * 16 + l16;
        const int n = n0 + wn * 128 + j * 16 + 4 * lq;
        float* p = resid + (size_t)m * N + n;
        const f32x4 v = old[ii][j] + acc[i2 + ii][j];
        if (m < M && vec && n + 3 < N) *reinterpret_cast<f32x4*>(p) = v;
        else
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (m < M && n + r < N) p[r] = v[r];
      }
  }
}

template <int EPI>
__global__ void __launch_bounds__(NWAVE * 64, 1)
k_gemm_mfma(const bf16* __restrict__ A, const bf16* __restrict__ W, int M, int N, int K,
            void* __restrict__ outv, float* __restrict__ resid, int tiles_m, int tiles_n, RopeAppend rp) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  typedef __attribute__((address_space(3))) void lds_void;
  constexpr bool GLU = (EPI == EPI_SWIGLU);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l16 = lane & 15, lq = lane >> 4;

  // ---- workgroup id -> tiles.  256 workgroups, one per CU (a workgroup's LDS fills a CU), each
  // walking tiles l, l + 256, l + 512, ...  Workgroup ids congruent modulo 8 land on the same
  // XCD, and its 32 workgroups take 32 consecutive tiles at a time.  Tile order, two levels:
  // groups of 16 tile rows; inside a group, columns of 8 tiles; inside a column, patches of 4
  // rows, row index fastest.  32 consecutive tiles are a 4 x 8 patch whose operand panels the
  // XCD's L2 shares, 256 consecutive tiles (what the eight XCDs work on at the same time) a
  // 16 x 16 block of the output.
  const int nt = tiles_m * tiles_n;
  int l = ((blockIdx.x & 7) << 5) + (blockIdx.x >> 3);
  if (l >= nt) return;
  TileAt ta = tile_at(l, tiles_m, tiles_n);
  bool has_next = l + PERSISTENT_WGS < nt;
  TileAt tb = tile_at(has_next ? l + PERSISTENT_WGS : l, tiles_m, tiles_n);  // the tile after this one
  int m0 = ta.tm * BM;
  int n0 = GLU ? ta.tn * (BN / 2) : ta.tn * BN;  // GLU: 128 output columns per tile

  // ---- global -> LDS: wave w fills tile rows 64w..64w+63 of both operands, 8 rows per
  // instruction; lane l supplies row 64w + 8i + l/8, physical chunk l%8.  Byte offsets from
  // the operand's base (both operands are below 4 GB): the k-block's offset is added to the
  // scalar base, so a fill costs no vector address arithmetic.
  unsigned ao[FI], wo[FI];
  auto fill_offsets = [&](const TileAt& t) {
    const int tm0 = t.tm * BM, tn0 = GLU ? t.tn * (BN / 2) : t.tn * BN;
    // (the lane number passes through an empty asm statement so that what is derived from it
    // is computed here, once per tile, instead of living in registers through the k-loop)
    int ln = lane;
    asm volatile("" : "+v"(ln));
#pragma unroll
    for (int i = 0; i < FI; ++i) {
      const int row = wave * 64 + i * 8 + (ln >> 3);
      const int c = (ln & 7) ^ ((row >> 1) & 7);
      const int am = min(tm0 + row, M - 1);
      ao[i] = (unsigned)(((size_t)am * K + c * 8) * 2);
      int wrow;
      if constexpr (GLU) {
        // tile row -> weight row: 32-row blocks alternate gate / up, so that a wave's 64 tile
        // rows are the gate and the up projection of the same 32 output columns
        const int blk = row >> 5;
        const int f = min(tn0 + (blk >> 1) * 32 + (row & 31), N - 1);
        wrow = (blk & 1) * N + f;
      } else {
        wrow = min(tn0 + row, N - 1);
      }
      wo[i] = (unsigned)(((size_t)wrow * K + c * 8) * 2);
    }
  };
  fill_offsets(ta);
  const int fill_off = wave * 64 * ROWB;
#define LS_FA(stage_, k0_, i_)                                                                        \
  __builtin_amdgcn_global_load_lds((const void*)((const char*)A + (size_t)(k0_) * 2 + ao[i_]),        \
      (lds_void*)(smem + (stage_) * STAGE_BYTES + fill_off + (i_) * 1024), 16, 0, 0);
#define LS_FW(stage_, k0_, i_)                                                                        \
  __builtin_amdgcn_global_load_lds((const void*)((const char*)W + (size_t)(k0_) * 2 + wo[i_]),        \
      (lds_void*)(smem + (stage_) * STAGE_BYTES + TILE_BYTES + fill_off + (i_) * 1024), 16, 0, 0);
  // both stages are free when a workgroup starts: stage 0 <- k-block 0 and stage 1 <- k-block 1
  // of its first tile at once (K >= 2 k-blocks); everything up to the first hand-over is set
  // up while these fills are on their way
#pragma unroll
  for (int i = 0; i < FI; ++i) {
    LS_FA(0, 0, i)
    LS_FW(0, 0, i)
  }
#pragma unroll
  for (int i = 0; i < FI; ++i) {
    LS_FA(1, BK, i)
    LS_FW(1, BK, i)
  }

  // ---- L2 prefetch.  A weight panel is shared by the 4 workgroups of a patch column, an
  // activation panel by the 8 of a patch row; whoever asks first waits for HBM or the
  // memory-side cache, and with two LDS stages a fill has one k-step to land.  So every
  // workgroup touches its share of the patch's lines PF_AHEAD k-steps before they are filled:
  // 64 of the 256 weight rows and 32 of the 256 activation rows, i.e. 16 + 8 lines per wavefront
  // and k-step, fetched by one 4-byte LDS-direct load (its lanes share those 24 lines; the
  // words go to a scratch piece of LDS nobody reads).  It is the youngest vector memory
  // operation of the wavefront at every hand-over, which therefore waits for all but one
  // (vmcnt(1)): vector memory loads return in order.  Measured at the 13B shape (with the
  // eight-wavefront version): the waits for fills at the hand-over (300-700 cycles per k-step
  // without it) disappear, +4.4 %.
  // The last k-steps of a tile prefetch the first k-blocks of the workgroup's next tile.
  auto pf_base = [&](const TileAt& t) -> const char* {
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int p = (ln & 31) < 24 ? (ln & 31) : (ln & 15);  // 24 distinct lines per wavefront
    const int row_w = (t.full ? 64 * t.q4 : 0) + 16 * wave + (p & 15);
    const int row_a = (t.full ? 32 * t.q8 : 0) + 8 * wave + (p & 7);
    const int tn0 = GLU ? t.tn * (BN / 2) : t.tn * BN;
    int wrow;
    if constexpr (GLU) {
      const int blk = row_w >> 5;
      const int f = min(tn0 + (blk >> 1) * 32 + (row_w & 31), N - 1);
      wrow = (blk & 1) * N + f;
    } else {
      wrow = min(tn0 + row_w, N - 1);
    }
    const int am = min(t.tm * BM + row_a, M - 1);
    return (p < 16) ? (const char*)W + (size_t)wrow * K * 2 : (const char*)A + (size_t)am * K * 2;
  };
  const char* pf_ptr = pf_base(ta);
  const char* pf_next = has_next ? pf_base(tb) : pf_ptr;
#define LS_PREFETCH(kb_)                                                                            \
  __builtin_amdgcn_global_load_lds(                                                                 \
      (const void*)((kb_) < KT ? pf_ptr + (size_t)(kb_) * (BK * 2)                                  \
                               : pf_next + (size_t)min((kb_) - KT, KT - 1) * (BK * 2)),             \
      (lds_void*)(smem + SMEM_BYTES), 4, 0, 0);
  f32x4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- LDS addresses of this lane's fragment reads in stage 0: fragment = 16 tile rows x 32 k,
  // lane -> row lane%16, k-octet lane/16 (first half-step) or 4 + lane/16 (second); later row
  // and column blocks are +2048 bytes (the swizzle term depends on row%16 only), stage 1 is
  // +STAGE_BYTES
  const unsigned lds0 = (unsigned)(size_t)(lds_void*)smem;
  const unsigned xa0 = lds0 + swz(wm * 128 + l16, lq), xa1 = lds0 + swz(wm * 128 + l16, 4 + lq);
  const unsigned wa0 = lds0 + TILE_BYTES + swz(wn * 128 + l16, lq);
  const unsigned wa1 = lds0 + TILE_BYTES + swz(wn * 128 + l16, 4 + lq);
  const int KT = K / BK;

  bf16x8 xf[2][8], wf[2][8];
#define LS_SB() __builtin_amdgcn_sched_barrier(0);
#define LS_RD(dst_, addr_, off_) \
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst_) : "v"(addr_), "n"(off_));
  // wait until at most n_ of this wavefront's LDS reads are outstanding (other counters untouched)
#define LS_WAITL(n_) __builtin_amdgcn_s_waitcnt(0xC07F | ((n_) << 8));
#define LS_MF(ws_, i_, j_) \
  acc[i_][j_] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[ws_][j_], xf[ws_][i_], acc[i_][j_], 0, 0, 0);
#define LS_NONE
  // two MFMAs, then one memory instruction (or none)
#define LS_MM(ws_, i_, j_, OP_) LS_MF(ws_, i_, j_) LS_SB() LS_MF(ws_, i_, (j_) + 1) LS_SB() OP_ LS_SB()
  // one row block of a half-step: eight MFMAs, a memory instruction after every second
#define LS_ROWB(ws_, i_, O0, O1, O2, O3) \
  LS_MM(ws_, i_, 0, O0) LS_MM(ws_, i_, 2, O1) LS_MM(ws_, i_, 4, O2) LS_MM(ws_, i_, 6, O3)
  // The fragments of a half-step are requested during the half-step before it, into the other
  // register set, always in the order W0 .. W7, X0 .. X7; LDS reads return in order.
  // First half-step of a k-step: its fragments were requested during the previous second
  // half-step, two per row block; the second half-step's fragments (k-octets 4..7 of the same
  // stage) are requested during row blocks 0..3, four per row block, so that the last of them
  // is 32 MFMAs old at the hand-over.  Row block 0 needs W0..W7 and X0: seven younger reads may
  // be outstanding.  Row block i needs X_i: 7 - i older-issued ones plus the 4 i requested in
  // this half-step so far, at most 15 (the counter's range; from row block 4 on the wait for
  // "at most 15" already covers X4..X7).
#define LS_HALF0(xaddr_, waddr_)                                                                          \
  LS_WAITL(7) LS_SB()                                                                                     \
  LS_ROWB(0, 0, LS_RD(wf[1][0], waddr_, 0 * 2048), LS_RD(wf[1][1], waddr_, 1 * 2048),                     \
          LS_RD(wf[1][2], waddr_, 2 * 2048), LS_RD(wf[1][3], waddr_, 3 * 2048))                           \
  LS_WAITL(10) LS_SB()                                                                                    \
  LS_ROWB(0, 1, LS_RD(wf[1][4], waddr_, 4 * 2048), LS_RD(wf[1][5], waddr_, 5 * 2048),                     \
          LS_RD(wf[1][6], waddr_, 6 * 2048), LS_RD(wf[1][7], waddr_, 7 * 2048))                           \
  LS_WAITL(13) LS_SB()                                                                                    \
  LS_ROWB(0, 2, LS_RD(xf[1][0], xaddr_, 0 * 2048), LS_RD(xf[1][1], xaddr_, 1 * 2048),                     \
          LS_RD(xf[1][2], xaddr_, 2 * 2048), LS_RD(xf[1][3], xaddr_, 3 * 2048))                           \
  LS_WAITL(15) LS_SB()                                                                                    \
  LS_ROWB(0, 3, LS_RD(xf[1][4], xaddr_, 4 * 2048), LS_RD(xf[1][5], xaddr_, 5 * 2048),                     \
          LS_RD(xf[1][6], xaddr_, 6 * 2048), LS_RD(xf[1][7], xaddr_, 7 * 2048))                           \
  LS_WAITL(15) LS_SB()                                                                                    \
  LS_ROWB(0, 4, LS_NONE, LS_NONE, LS_NONE, LS_NONE)                                                       \
  LS_ROWB(0, 5, LS_NONE, LS_NONE, LS_NONE, LS_NONE)                                                       \
  LS_ROWB(0, 6, LS_NONE, LS_NONE, LS_NONE, LS_NONE)                                                       \
  LS_ROWB(0, 7, LS_NONE, LS_NONE, LS_NONE, LS_NONE)
  // Second half-step: its fragments all arrived before the hand-over.  Per row block two
  // requests for the next k-step's first half-step (k-octets 0..3 of the other stage) and two
  // fills of the retired stage; the L2 prefetch goes last.
#define LS_HALF1(xaddr_, waddr_, stage_, k2_, PF_)                                                        \
  LS_ROWB(1, 0, LS_RD(wf[0][0], waddr_, 0 * 2048), LS_FA(stage_, k2_, 0), LS_RD(wf[0][1], waddr_, 1 * 2048), LS_FW(stage_, k2_, 0)) \
  LS_ROWB(1, 1, LS_RD(wf[0][2], waddr_, 2 * 2048), LS_FA(stage_, k2_, 1), LS_RD(wf[0][3], waddr_, 3 * 2048), LS_FW(stage_, k2_, 1)) \
  LS_ROWB(1, 2, LS_RD(wf[0][4], waddr_, 4 * 2048), LS_FA(stage_, k2_, 2), LS_RD(wf[0][5], waddr_, 5 * 2048), LS_FW(stage_, k2_, 2)) \
  LS_ROWB(1, 3, LS_RD(wf[0][6], waddr_, 6 * 2048), LS_FA(stage_, k2_, 3), LS_RD(wf[0][7], waddr_, 7 * 2048), LS_FW(stage_, k2_, 3)) \
  LS_ROWB(1, 4, LS_RD(xf[0][0], xaddr_, 0 * 2048), LS_FA(stage_, k2_, 4), LS_RD(xf[0][1], xaddr_, 1 * 2048), LS_FW(stage_, k2_, 4)) \
  LS_ROWB(1, 5, LS_RD(xf[0][2], xaddr_, 2 * 2048), LS_FA(stage_, k2_, 5), LS_RD(xf[0][3], xaddr_, 3 * 2048), LS_FW(stage_, k2_, 5)) \
  LS_ROWB(1, 6, LS_RD(xf[0][4], xaddr_, 4 * 2048), LS_FA(stage_, k2_, 6), LS_RD(xf[0][5], xaddr_, 5 * 2048), LS_FW(stage_, k2_, 6)) \
  LS_ROWB(1, 7, LS_RD(xf[0][6], xaddr_, 6 * 2048), LS_FA(stage_, k2_, 7), LS_RD(xf[0][7], xaddr_, 7 * 2048), LS_FW(stage_, k2_, 7) PF_)
  // own LDS reads done, own fills landed, then everyone
#define LS_HANDOVER(imm_)                    \
  asm volatile("" ::: "memory");             \
  __builtin_amdgcn_s_waitcnt(imm_);          \
  __builtin_amdgcn_sched_barrier(0);         \
  __builtin_amdgcn_s_barrier();              \
  __builtin_amdgcn_sched_barrier(0);         \
  asm volatile("" ::: "memory");

  // first fragments of a tile: k-octets 0..3 of the stage at byte offset so_
#define LS_FIRST_READS(so_)                                                                            \
  LS_SB()                                                                                              \
  LS_RD(wf[0][0], wa0 + (so_), 0 * 2048) LS_RD(wf[0][1], wa0 + (so_), 1 * 2048)                        \
  LS_RD(wf[0][2], wa0 + (so_), 2 * 2048) LS_RD(wf[0][3], wa0 + (so_), 3 * 2048)                        \
  LS_RD(wf[0][4], wa0 + (so_), 4 * 2048) LS_RD(wf[0][5], wa0 + (so_), 5 * 2048)                        \
  LS_RD(wf[0][6], wa0 + (so_), 6 * 2048) LS_RD(wf[0][7], wa0 + (so_), 7 * 2048)                        \
  LS_RD(xf[0][0], xa0 + (so_), 0 * 2048) LS_RD(xf[0][1], xa0 + (so_), 1 * 2048)                        \
  LS_RD(xf[0][2], xa0 + (so_), 2 * 2048) LS_RD(xf[0][3], xa0 + (so_), 3 * 2048)                        \
  LS_RD(xf[0][4], xa0 + (so_), 4 * 2048) LS_RD(xf[0][5], xa0 + (so_), 5 * 2048)                        \
  LS_RD(xf[0][6], xa0 + (so_), 6 * 2048) LS_RD(xf[0][7], xa0 + (so_), 7 * 2048)                        \
  LS_SB()
  // ---- prologue: prefetch, hand over stage 0 (the sixteen fills of stage 1 and the prefetch
  // may still be in flight: vmcnt(17), whose upper bits sit in bits 15:14 of the immediate),
  // first fragments
  LS_PREFETCH(1 + PF_AHEAD)
  LS_HANDOVER(0x4071)
  LS_FIRST_READS(0u)

  // The workgroup's k-steps form one stream across its tiles: stage = (k-steps so far) & 1, and
  // the fills of a tile's last two k-steps already fetch the first two k-blocks of the
  // workgroup's next tile, so that its epilogue, not an idle CU, covers their latency.
  int kf = 2;       // next k-block to fetch, of the tile that ao/wo point at
  unsigned gk = 0;  // k-steps done
  for (;;) {
    for (int kt = 0; kt < KT; ++kt, ++gk) {
      const int buf = gk & 1;
      const unsigned sx = (unsigned)buf * STAGE_BYTES, so = (unsigned)(buf ^ 1) * STAGE_BYTES;
      // first half-step: computes k-octets 0..3 of stage buf, requests octets 4..7 of the same stage
      {
        const unsigned xa = xa1 + sx, wa = wa1 + sx;
        LS_SB()
        LS_HALF0(xa, wa)
      }
      // vmcnt(1): all fills, not the youngest prefetch.  (Right after an epilogue this also waits
      // for all but the last of its stores; a hand-over that lets them pass, with the fills
      // waited for before the epilogue instead, measured 1-2 % slower in the residual GEMMs.)
      LS_HANDOVER(0x0071)
      // second half-step: computes octets 4..7, requests octets 0..3 of the other stage and
      // refills stage buf
      {
        if (kf == KT) {
          // nothing left to fetch for this tile: go on with the next one's first k-blocks; the
          // very last tile fills the retired stage once more with its last k-block (lines that
          // are in L2 anyway) instead of branching around every fill
          if (has_next) {
            // (computed here, from two scalars, rather than a whole tile ahead of their use:
            // the compiler would otherwise keep sixteen more registers alive through the k-loop)
            asm volatile("" : "+s"(tb.tm), "+s"(tb.tn));
            fill_offsets(tb);
            kf = 0;
          } else {
            kf = KT - 1;
          }
        }
        const unsigned xa = xa0 + so, wa = wa0 + so;
        const int k2 = kf * BK;
        ++kf;
        LS_SB()
        LS_HALF1(xa, wa, buf, k2, LS_PREFETCH(kt + 2 + PF_AHEAD))
      }
    }
    // the fragments requested by the last half-step land in registers the epilogue may reuse:
    // wait for them (LDS reads only; fills stay in flight), and request them again afterwards
    LS_SB()
    LS_WAITL(0)
    LS_SB()
    if constexpr (EPI == EPI_RESID) {
      add_tile_to_residual(acc, m0, n0, M, N, resid, wm, wn, l16, lq);
    } else if constexpr (EPI == EPI_F32) {
      store_tile_f32(acc, m0, n0, M, N, (float*)outv, wm, wn, l16, lq);
    } else {
      store_tile<EPI, 0>(acc, m0, n0, M, N, outv, resid, rp, wm, 2 * wn, l16, lq);
      store_tile<EPI, 4>(acc, m0, n0, M, N, outv, resid, rp, wm, 2 * wn + 1, l16, lq);
    }
    if (!has_next) break;
    l += PERSISTENT_WGS;
    ta = tb;
    has_next = l + PERSISTENT_WGS < nt;
    tb = tile_at(has_next ? l + PERSISTENT_WGS : l, tiles_m, tiles_n);
    m0 = ta.tm * BM;
    n0 = GLU ? ta.tn * (BN / 2) : ta.tn * BN;
    pf_ptr = pf_next;
    pf_next = has_next ? pf_base(tb) : pf_ptr;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    // the new tile's first k-block landed before the hand-over of the last k-step
    LS_FIRST_READS((unsigned)(gk & 1) * STAGE_BYTES)
  }
  // no LDS-direct load may still be on its way when the workgroup gives up its LDS
  LS_SB()
  __builtin_amdgcn_s_waitcnt(0x0070);
  LS_SB()
#undef LS_FIRST_READS
#undef LS_FA
#undef LS_FW
#undef LS_SB
#undef LS_RD
#undef LS_WAITL
#undef LS_MF
#undef LS_NONE
#undef LS_MM
#undef LS_ROWB
#undef LS_HALF0
#undef LS_HALF1
#undef LS_HANDOVER
#undef LS_PREFETCH

}

template <int EPI>
void launch_t(const void* A, const void* W, int M, int N, int K, void* out, float* resid, hipStream_t st,
              const RopeAppend& rope = RopeAppend{}) {
  static std::atomic<uint64_t> lds_allowed{0};
  constexpr int LDS_BYTES = SMEM_BYTES + 256;  // + the scratch words of the L2 prefetch
  allow_dynamic_lds((const void*)k_gemm_mfma<EPI>, LDS_BYTES, lds_allowed);
  const int tiles_m = (M + BM - 1) / BM;
  const int ncols = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  const int tiles_n = (N + ncols - 1) / ncols;
  const int nt = tiles_m * tiles_n;
  (void)nt;
  const int grid = PERSISTENT_WGS;  // workgroups whose first tile does not exist leave at once
  launch_kernel(k_gemm_mfma<EPI>, dim3(grid), dim3(NWAVE * 64), LDS_BYTES, st, (const bf16*)A, (const bf16*)W, M, N,
                K, out, resid, tiles_m, tiles_n, rope);
}

}  // namespace

bool gemm_mfma_supported(int M, int N, int K) { return M >= 1 && N >= 1 && K >= 2 * BK && K % BK == 0; }

bool gemm_mfma_rope_supported(int M, int N, int K, int hq, int hkv, int hd) {
  return gemm_mfma_supported(M, N, K) && (hd == 64 || hd == 128) && N == (hq + 2 * hkv) * hd;
}

void launch_gemm_mfma_rope(const void* A, const void* W, int M, int N, int K, void* out, const RopeAppend& rope,
                           hipStream_t st) {
  launch_t<EPI_ROPE>(A, W, M, N, K, out, nullptr, st, rope);
}

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

