// bf16 causal attention for the prompt pass (flash-style, MFMA, K/V tiles staged in LDS).
//
// One 256-thread workgroup handles 128 consecutive query rows of one (sequence, query head);
// each of its 4 wavefronts owns 32 rows and keeps them, the running maximum, the running sum
// and the output accumulator in registers while the workgroup walks the keys 0..last row in
// tiles of 64, double-buffered in LDS.  Both products are computed transposed so that all
// per-row softmax state is per-lane:
//   S^T[key][q] = K[key][:] . Q[q][:]      MFMA A = K tile rows,  B = Q rows (registers)
//   O^T[d][q]  += V^T[d][key] . P^T[key][q] MFMA A = V^T,          B = P^T
// In a v_mfma_f32_32x32x16_bf16 result a lane holds column q = lane%32 and 16 rows
// 8*(i/4) + 4*(lane/32) + i%4: one query row per lane, so the row maximum / sum are
// in-lane reductions plus one exchange with lane^32, and the eight P values a lane holds
// for a 16-key step are exactly a B operand whose k index runs over keys
// {4h..4h+3, 8+4h..8+4h+3} (h = lane/32).
//
// K and V tiles lie in LDS as they lie in the cache, row-major [key][head_dim], and arrive
// there straight from global memory (global_load_lds_dwordx4: no staging registers, no LDS
// store instructions).  The V^T operand is produced by the LDS read itself: with
// ds_read_b64_tr_b16 the 16 lanes of a group hand in the addresses of a 4-key x 16-dim block
// (lane j: key j/4, dims 4(j%4)..4(j%4)+3) and lane j receives that block's column j, i.e.
// the four keys' values at ONE dim -- half an A operand of V^T in the key order above; two such
// reads make one operand.  16-byte chunks of a row are XOR-swizzled by a permutation of the
// key's low bits chosen so that both access patterns spread over all banks: the 32 rows of a
// K operand read (one 16-byte chunk per row) and the 4 rows x 32 bytes of a transposing read.
//
// A wavefront whose 32 rows all lie above a key tile skips that tile's arithmetic (it still
// takes part in the fills and barriers); the output rescale is skipped when no row's running
// maximum moved.  Keys beyond a row's position get a score of -inf before the exponential;
// cache rows at or beyond the sequence length are never read (indices are clamped).
#include "kernels.hpp"
#include "device_util.hpp"

namespace ls {

namespace {

constexpr int BQ = 128, BKV = 64;

template <int HD>
__global__ void __launch_bounds__(256, 2)
k_attn_prefill(const bf16* __restrict__ qkv, int qkv_stride, const bf16* __restrict__ kc,
               const bf16* __restrict__ vc, const int32_t* __restrict__ cu, int hq, int hkv, int max_seq,
               bf16* __restrict__ out, int nq, int batch) {
  constexpr int ROWB = HD * 2;            // bytes per K / V row
  constexpr int CPR = HD / 8;             // 16-byte chunks per row: 16 or 8
  constexpr int TILE = BKV * ROWB;        // one K or V tile
  constexpr int RPI = 1024 / ROWB;        // rows one fill instruction covers: 4 or 8
  constexpr int FI = BKV / (4 * RPI);     // fill instructions per wavefront, tile and operand
  constexpr int DT = HD / 32;             // 32-row tiles of O^T
  constexpr int KS = HD / 16;             // k-steps of the score product
  __shared__ __attribute__((aligned(1024))) unsigned char smem[2][2 * TILE];
  typedef __attribute__((address_space(3))) void lds_void;
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

  // Workgroup id -> (sequence, head, query tile).  All query tiles of all heads that share one
  // (sequence, kv head) read the same keys and values, several times over (a causal prefix
  // each).  Workgroup ids congruent modulo 8 run on the same XCD, so the nq * G workgroups of
  // such a group get ids that are 8 apart: they run side by side behind one L2 and the group's
  // keys and values come from memory once (with consecutive ids, the eight query tiles of a
  // head ran on eight XCDs and each fetched its own copy: 2.5 x the algorithmic bytes).
  // Within a group: longest query tiles first, the G heads of a tile next to each other.
  const int G = hq / hkv;
  const int ngroup = batch * hkv;
  int grp, t;
  if ((ngroup & 7) == 0) {
    const int j = blockIdx.x >> 3;
    t = j % (nq * G);
    grp = (j / (nq * G)) * 8 + (blockIdx.x & 7);
  } else {
    t = blockIdx.x % (nq * G);
    grp = blockIdx.x / (nq * G);
  }
  const int b = grp / hkv, kh = grp % hkv;
  const int h = kh * G + t % G;
  const int row0 = cu[b], len = cu[b + 1] - row0;
  const int ntile = (len + BQ - 1) / BQ;
  const int qt = ntile - 1 - t / G;  // longest tiles first
  if (qt < 0) return;
  const int q0 = qt * BQ;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: what depends on it is wave-uniform
  const int lr = lane & 31, lh = lane >> 5;
  const bf16* kb = kc + ((size_t)b * hkv + kh) * max_seq * HD;
  const bf16* vb = vc + ((size_t)b * hkv + kh) * max_seq * HD;

  // chunk swizzle of row `key`: a permutation of the key's low bits (see the file header)
  auto swz = [](int key) { return HD == 128 ? (((key & 3) << 2) | ((key >> 2) & 3)) : (((key & 3) << 1) | ((key >> 2) & 1)); };

  // this lane's query row as B operands (one 8-wide k slice per k-step)
  const int qpos = q0 + wave * 32 + lr;            // position of this lane's query row
  const int qrow = row0 + min(qpos, len - 1);      // clamped: rows past the end are discarded
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(qkv + (size_t)qrow * qkv_stride + (size_t)h * HD + ks * 16 + lh * 8);

  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;  // l_run: this lane's half of the row sum
  const float c = 1.4426950408889634f / sqrtf((float)HD);  // score -> exponent of 2

  const int kv_end = min(q0 + BQ, len);          // keys this tile can see
  const int ntk = (kv_end + BKV - 1) / BKV;
  const int wave_last = q0 + wave * 32 + 31;     // last position any row of this wavefront has

  // ---- fills: wavefront w brings rows (w*FI + i)*RPI .. +RPI-1 of both tiles; the lane that
  // fills physical chunk p of row r fetches logical chunk p ^ swz(r)
  const int frow = lane / CPR, fchunk = lane % CPR;
#define LS_FILL(buf, t0)                                                                          \
  _Pragma("unroll") for (int i_ = 0; i_ < FI; ++i_) {                                             \
    const int r_ = (wave * FI + i_) * RPI + frow;                                                 \
    const size_t g_ = (size_t)min((t0) + r_, len - 1) * HD + ((fchunk ^ swz(r_)) << 3);            \
    __builtin_amdgcn_global_load_lds((const void*)(kb + g_),                                      \
        (lds_void*)(smem[buf] + (wave * FI + i_) * 1024), 16, 0, 0);                              \
    __builtin_amdgcn_global_load_lds((const void*)(vb + g_),                                      \
        (lds_void*)(smem[buf] + TILE + (wave * FI + i_) * 1024), 16, 0, 0);                       \
  }
  // all fills this wavefront issued have landed, then the workgroup meets
#define LS_TILE_BARRIER()                    \
  asm volatile("" ::: "memory");             \
  __builtin_amdgcn_s_waitcnt(0x0F70);        \
  __builtin_amdgcn_s_waitcnt(0xC07F);        \
  __builtin_amdgcn_sched_barrier(0);         \
  __builtin_amdgcn_s_barrier();              \
  __builtin_amdgcn_sched_barrier(0);         \
  asm volatile("" ::: "memory");

  // LDS byte offsets of this lane's operand reads inside a tile
  const int ksw = swz(lr);                        // rows lr and 32 + lr share their low bits
  const int k_row = lr * ROWB;
  // transposing read: group g = lane/16 covers dims 16*(g&1).., keys 4*(g>>1) + j/4; lane j of
  // the group addresses dims 4*(j%4)..+3 of its key
  const int tj = lane & 15, tg = lane >> 4;
  const int v_key = 4 * (tg >> 1) + (tj >> 2);    // + 16 kp (+ 8 for the second half)
  const int v_col = 16 * (tg & 1) + 4 * (tj & 3);  // + 32 dt: first dim this lane addresses
  const int v_sub = (v_col & 7) * 2;              // byte offset inside its 16-byte chunk

  LS_FILL(0, 0)
  LS_TILE_BARRIER()
  for (int t = 0; t < ntk; ++t) {
    const int buf = t & 1;
    const int t0 = t * BKV;
    // buffer buf^1 was last read in iteration t-1, which every wavefront has left
    if (t + 1 < ntk) LS_FILL(buf ^ 1, t0 + BKV)
    const unsigned char* ks_ = smem[buf];
    const unsigned char* vs_ = smem[buf] + TILE;

    if (t0 <= wave_last) {  // wave-uniform: some row of this wavefront sees some key of the tile
      // ---- S^T = K Q^T for the 64 keys of the tile (two 32-key row tiles)
      f32x16 s[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kt][i] = 0.f;
#pragma unroll
        for (int ksn = 0; ksn < KS; ++ksn) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks_ + kt * 32 * ROWB + k_row + (((ksn * 2 + lh) ^ ksw) << 4));
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ksn], s[kt], 0, 0, 0);
        }
      }
      // ---- causal mask, online softmax (all for this lane's query row).  Scores stay unscaled:
      // the running maximum is kept in score units and the scale (with the change to base 2)
      // is folded into the exponential's argument, p = 2^(c s - c m).
      // `diag` is the same for the whole wavefront: tiles left of the diagonal skip the mask.
      const bool diag = (t0 + BKV - 1) > (q0 + wave * 32);
      float mx = -INFINITY;
      if (diag) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = t0 + kt * 32 + 8 * (i >> 2) + 4 * lh + (i & 3);
            const float v = key > qpos ? -INFINITY : s[kt][i];
            s[kt][i] = v;
            mx = fmaxf(mx, v);
          }
      } else {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kt][i]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);  // finite from the first tile on: key 0 is visible
      const float mc = m_new * c;
      float psum = 0.f;
      bf16x8 pf[4];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[kt][i], c, -mc));
          psum += p;
          pf[kt * 2 + (i >> 3)][i & 7] = (bf16)p;
        }
      // the running maximum moved for some row of the wavefront: rescale sums and outputs
      if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
        const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * c);
        l_run *= corr;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[dt][i] *= corr;
        m_run = m_new;
      }
      l_run += psum;
      // ---- O^T += V^T P^T; the V^T operand comes out of two transposing reads
#pragma unroll
      for (int kp = 0; kp < 4; ++kp) {  // 16-key steps
        const int key0 = 16 * kp + v_key, key1 = key0 + 8;
        const int sw0 = swz(key0), sw1 = swz(key1);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const int ch = (32 * dt + v_col) >> 3;  // logical 16-byte chunk of the addressed dims
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (lds_s16x4*)(vs_ + key0 * ROWB + ((ch ^ sw0) << 4) + v_sub));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (lds_s16x4*)(vs_ + key1 * ROWB + ((ch ^ sw1) << 4) + v_sub));
          typedef short s16x8 __attribute__((ext_vector_type(8)));
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[kp], o[dt], 0, 0, 0);
        }
      }
    }
    LS_TILE_BARRIER()
  }
#undef LS_FILL
#undef LS_TILE_BARRIER

  // ---- normalise and store this lane's query row
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_tot;
  if (qpos < len) {
    bf16* orow = out + (size_t)(row0 + qpos) * ((size_t)hq * HD) + (size_t)h * HD;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[dt][g * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + dt * 32 + 8 * g + 4 * lh) = v;
      }
  }
}

}  // namespace

bool attn_prefill_supported(int hq, int hkv, int hd) { return (hd == 128 || hd == 64) && hq % hkv == 0; }

void launch_attn_prefill(const void* qkv, int qkv_stride, const void* kc, const void* vc, const int32_t* cu_seqlens,
                         int batch, int max_len, int hq, int hkv, int hd, int max_seq, void* out, hipStream_t st) {
  if (batch <= 0 || max_len <= 0) return;
  const int nq = (max_len + BQ - 1) / BQ;
  dim3 grid((unsigned)nq * hq * batch);
  if (hd == 128)
    k_attn_prefill<128><<<grid, 256, 0, st>>>((const bf16*)qkv, qkv_stride, (const bf16*)kc, (const bf16*)vc,
                                              cu_seqlens, hq, hkv, max_seq, (bf16*)out, nq, batch);
  else
    k_attn_prefill<64><<<grid, 256, 0, st>>>((const bf16*)qkv, qkv_stride, (const bf16*)kc, (const bf16*)vc,
                                             cu_seqlens, hq, hkv, max_seq, (bf16*)out, nq, batch);
}

}  // namespace ls
