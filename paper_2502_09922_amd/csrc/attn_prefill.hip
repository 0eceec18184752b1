// bf16 causal attention for the prompt pass (flash-style, MFMA, K/V tiles staged in LDS).
//
// One 256-thread workgroup handles 128 consecutive query rows of one (sequence, query head);
// each of its 4 wavefronts owns 32 rows and keeps them, the running maximum, the running sum
// and the output accumulator in registers while the workgroup walks the keys 0..last row in
// tiles of 64, double-buffered in LDS.  Both products are computed transposed so that all
// per-row softmax state is per-lane:
//   S^T[key][q] = K[key][:] . Q[q][:]      MFMA A = K tile rows,  B = Q rows (registers)
//   O^T[d][q]  += V^T[d][key] . P^T[key][q] MFMA A = V^T tile rows, B = P^T
// In a v_mfma_f32_32x32x16_bf16 result a lane holds column q = lane%32 and 16 rows
// 8*(i/4) + 4*(lane/32) + i%4: one query row per lane, so the row maximum / sum are
// in-lane reductions plus one exchange with lane^32, and the eight P values a lane holds
// for a 16-key step are exactly a B operand whose k index runs over keys
// {4h..4h+3, 8+4h..8+4h+3} (h = lane/32); the V^T operand is read with the same key order.
// V is transposed on its way into LDS ([d][key], 8-byte granules XOR-swizzled by d/2).
// Keys beyond a row's position get a score of -inf before the exponential; cache rows at or
// beyond the sequence length are never read (indices are clamped to the last valid row).
#include "kernels.hpp"
#include "device_util.hpp"

namespace ls {

namespace {

constexpr int BQ = 128, BKV = 64;

template <int HD>
__global__ void __launch_bounds__(256, 2)
k_attn_prefill(const bf16* __restrict__ qkv, int qkv_stride, const bf16* __restrict__ kc,
               const bf16* __restrict__ vc, const int32_t* __restrict__ cu, int hq, int hkv, int max_seq,
               bf16* __restrict__ out) {
  constexpr int CPR = HD / 8;            // 16-byte chunks per K row
  constexpr int KT_BYTES = BKV * HD * 2;  // K tile; the V^T tile has the same size
  constexpr int KLD = (BKV * CPR) / 256;  // K chunks per thread per tile
  constexpr int VLD = (32 * CPR) / 256;   // V work items (key pair x 8 dims) per thread per tile
  constexpr int DT = HD / 32;            // 32-row tiles of O^T
  constexpr int KS = HD / 16;            // k-steps of the score product
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][2 * KT_BYTES];

  const int b = blockIdx.z, h = blockIdx.y;
  const int row0 = cu[b], len = cu[b + 1] - row0;
  const int ntile = (len + BQ - 1) / BQ;
  const int qt = ntile - 1 - (int)blockIdx.x;  // longest tiles first
  if (qt < 0) return;
  const int q0 = qt * BQ;
  const int kh = h / (hq / hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lh = lane >> 5;
  const bf16* kb = kc + ((size_t)b * hkv + kh) * max_seq * HD;
  const bf16* vb = vc + ((size_t)b * hkv + kh) * max_seq * HD;

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

  // staging registers for the next K / V tile
  u32x4 kreg[KLD], vreg[VLD][2];
#define LS_LOAD_KV(t0)                                                                    \
  {                                                                                       \
    _Pragma("unroll") for (int i_ = 0; i_ < KLD; ++i_) {                                  \
      const int w_ = tid + 256 * i_;                                                      \
      const int key_ = min((t0) + w_ / CPR, len - 1);                                     \
      kreg[i_] = *reinterpret_cast<const u32x4*>(kb + (size_t)key_ * HD + (w_ % CPR) * 8); \
    }                                                                                     \
    _Pragma("unroll") for (int i_ = 0; i_ < VLD; ++i_) {                                  \
      const int w_ = tid + 256 * i_;                                                      \
      const int k0_ = (t0) + 2 * (w_ / CPR);                                              \
      vreg[i_][0] = *reinterpret_cast<const u32x4*>(vb + (size_t)min(k0_, len - 1) * HD + (w_ % CPR) * 8);     \
      vreg[i_][1] = *reinterpret_cast<const u32x4*>(vb + (size_t)min(k0_ + 1, len - 1) * HD + (w_ % CPR) * 8); \
    }                                                                                     \
  }
#define LS_STORE_KV(buf)                                                                  \
  {                                                                                       \
    unsigned char* ks_ = smem[buf];                                                       \
    unsigned char* vs_ = smem[buf] + KT_BYTES;                                            \
    _Pragma("unroll") for (int i_ = 0; i_ < KLD; ++i_) {                                  \
      const int w_ = tid + 256 * i_;                                                      \
      const int r_ = w_ / CPR, c_ = w_ % CPR;                                             \
      const int sw_ = (HD == 128) ? (r_ & 15) : ((r_ >> 1) & 7);                          \
      *reinterpret_cast<u32x4*>(ks_ + r_ * (HD * 2) + ((c_ ^ sw_) << 4)) = kreg[i_];      \
    }                                                                                     \
    _Pragma("unroll") for (int i_ = 0; i_ < VLD; ++i_) {                                  \
      const int w_ = tid + 256 * i_;                                                      \
      const int kp_ = w_ / CPR, dc_ = w_ % CPR;                                           \
      _Pragma("unroll") for (int e_ = 0; e_ < 8; ++e_) {                                  \
        const int d_ = dc_ * 8 + e_;                                                      \
        const unsigned lo_ = (vreg[i_][0][e_ >> 1] >> ((e_ & 1) * 16)) & 0xffffu;         \
        const unsigned hi_ = (vreg[i_][1][e_ >> 1] >> ((e_ & 1) * 16)) & 0xffffu;         \
        const int g_ = (kp_ >> 1) ^ ((d_ >> 1) & 15);                                     \
        *reinterpret_cast<unsigned*>(vs_ + d_ * 128 + g_ * 8 + (kp_ & 1) * 4) = lo_ | (hi_ << 16); \
      }                                                                                   \
    }                                                                                     \
  }

  LS_LOAD_KV(0)
  LS_STORE_KV(0)
  __syncthreads();
  for (int t = 0; t < ntk; ++t) {
    const int buf = t & 1;
    const int t0 = t * BKV;
    if (t + 1 < ntk) LS_LOAD_KV(t0 + BKV)
    const unsigned char* ks_ = smem[buf];
    const unsigned char* vs_ = smem[buf] + KT_BYTES;

    // ---- S^T = K Q^T for the 64 keys of the tile (two 32-key row tiles)
    f32x16 s[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kt][i] = 0.f;
      const int r = kt * 32 + lr;
      const int sw = (HD == 128) ? (r & 15) : ((r >> 1) & 7);
#pragma unroll
      for (int ksn = 0; ksn < KS; ++ksn) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks_ + r * (HD * 2) + (((ksn * 2 + lh) ^ sw) << 4));
        s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ksn], s[kt], 0, 0, 0);
      }
    }
    // ---- causal mask, online softmax (all for this lane's query row).  Scores stay unscaled:
    // the running maximum is kept in score units and the scale (with the change to base 2)
    // is folded into the exponential's argument, p = 2^(c s - c m).
    // `diag` is the same for the whole wavefront: tiles left of the diagonal skip the mask.
    const bool diag = __builtin_amdgcn_readfirstlane((int)((t0 + BKV - 1) > (q0 + wave * 32))) != 0;
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
    const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * c);
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
    l_run = l_run * corr + psum;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] *= corr;
    // ---- O^T += V^T P^T
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const int d = dt * 32 + lr;
      const int sw = (d >> 1) & 15;
#pragma unroll
      for (int kp = 0; kp < 4; ++kp) {  // 16-key steps
        bf16x4 lo = *reinterpret_cast<const bf16x4*>(vs_ + d * 128 + (((kp * 4 + lh) ^ sw) << 3));
        bf16x4 hi = *reinterpret_cast<const bf16x4*>(vs_ + d * 128 + (((kp * 4 + 2 + lh) ^ sw) << 3));
        bf16x8 vf;
#pragma unroll
        for (int e = 0; e < 4; ++e) { vf[e] = lo[e]; vf[4 + e] = hi[e]; }
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kp], o[dt], 0, 0, 0);
      }
    }
    if (t + 1 < ntk) LS_STORE_KV(buf ^ 1)
    __syncthreads();
  }
#undef LS_LOAD_KV
#undef LS_STORE_KV

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
  dim3 grid((max_len + BQ - 1) / BQ, hq, batch);
  if (hd == 128)
    k_attn_prefill<128><<<grid, 256, 0, st>>>((const bf16*)qkv, qkv_stride, (const bf16*)kc, (const bf16*)vc,
                                              cu_seqlens, hq, hkv, max_seq, (bf16*)out);
  else
    k_attn_prefill<64><<<grid, 256, 0, st>>>((const bf16*)qkv, qkv_stride, (const bf16*)kc, (const bf16*)vc,
                                             cu_seqlens, hq, hkv, max_seq, (bf16*)out);
}

}  // namespace ls
