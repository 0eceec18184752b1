// bf16 decode attention, fused with RoPE and the KV-cache append of the new row: one query
// row per sequence against its KV cache (GQA aware).
//
// The step's q, k, v are read un-rotated from the projection output.  q is rotated in
// registers; the new key is rotated, rounded to bf16 and written to the cache row `pos`
// together with the new value by wave 0, which also feeds them to its own softmax state
// straight from registers -- no wavefront of this kernel reads cache row `pos`, so there is
// no ordering problem between that store and the streaming loads.
//
// Bound by streaming the cache out of HBM once per step, so: one workgroup per (sequence,
// kv head) reads that head's keys and values exactly once for all G = Hq/Hkv query heads
// that share it.  Its NW wavefronts split the context into contiguous ranges (split-KV
// inside the workgroup).  A 16-byte-per-lane load instruction fetches 64/LPK consecutive
// cache rows (LPK = head_dim/8 lanes per key, whole rows, 1 KB contiguous).  Each lane
// keeps the partial dot product of its 8 dimensions, a butterfly over the LPK lanes of a key
// completes the score, and every key slot runs its own online softmax (running max and sum)
// so that no cross-slot traffic is needed inside the loop.  Slots are merged by shuffles,
// wavefronts through LDS in wave order: the result does not depend on timing.
#include "kernels.hpp"
#include "device_util.hpp"

namespace ls {

namespace {

// wavefronts per workgroup = context splits.  With one query head per kv head the kernel
// needs few registers and 16 wavefronts with one load per operand in flight stream best
// (measured inside the stage, 7B and 13B shapes); wider groups keep 8 wavefronts.
#ifndef LS_ATTN_NW
#define LS_ATTN_NW 8
#endif
#ifndef LS_ATTN_NW1
#define LS_ATTN_NW1 16
#endif
#ifndef LS_ATTN_U
#define LS_ATTN_U 1
#endif
constexpr int waves_for(int g) { return g == 1 ? LS_ATTN_NW1 : LS_ATTN_NW; }

template <int HD, int G>
// with one query head per kv head the kernel fits 64 registers: eight wavefronts per SIMD, two
// 16-wavefront workgroups per CU
__global__ void __launch_bounds__(waves_for(G) * 64, (G == 1 ? 8 : 1))
k_attn_decode(const bf16* __restrict__ qkv, int qkv_stride, const float2* __restrict__ cs,
              bf16* __restrict__ kc, bf16* __restrict__ vc, const int32_t* __restrict__ row_seq,
              const int32_t* __restrict__ row_pos, int hq, int hkv, int max_seq, bf16* __restrict__ out) {
  constexpr int NW = waves_for(G);
  constexpr int LPK = HD / 8;     // lanes per key
  constexpr int KPI = 64 / LPK;   // keys per load instruction
  constexpr int U = (G >= 4) ? 2 : LS_ATTN_U;  // load instructions in flight per operand
  __shared__ float sm_m[NW][G], sm_l[NW][G];
  __shared__ float sm_acc[NW][G][HD];
  const int r = blockIdx.x, kh = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pos = row_pos[r];
  if (pos < 0) return;  // a sequence with no room left: whole workgroup leaves together
  const int seq = row_seq[r];
  const int ctx = pos;  // keys 0..pos-1 come from the cache, key `pos` from this step's row
  const int slot = lane / LPK, dl = lane % LPK;
  bf16* kb = kc + ((size_t)seq * hkv + kh) * max_seq * HD;
  bf16* vb = vc + ((size_t)seq * hkv + kh) * max_seq * HD;
  const bf16* row = qkv + (size_t)r * qkv_stride;

  // cos/sin of this lane's four pairs (dims 8 dl + 2i, 8 dl + 2i + 1) at position pos
  float2 rot[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) rot[i] = cs[(size_t)pos * (HD / 2) + dl * 4 + i];

  // this lane's 8 dimensions of every query head of the group: rotated, pre-scaled
  const float scale = 1.0f / sqrtf((float)HD);
  float q[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const bf16x8 qv = *reinterpret_cast<const bf16x8*>(row + (size_t)(kh * G + g) * HD + dl * 8);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float u0 = (float)qv[2 * i], u1 = (float)qv[2 * i + 1];
      q[g][2 * i] = (u0 * rot[i].x - u1 * rot[i].y) * scale;
      q[g][2 * i + 1] = (u0 * rot[i].y + u1 * rot[i].x) * scale;
    }
  }

  // contiguous key range of this wave, a multiple of KPI keys
  const int chunk = ((ctx + NW * KPI - 1) / (NW * KPI)) * KPI;
  const int k_begin = wave * chunk, k_end = min(k_begin + chunk, ctx);

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
  }

  // one key per slot: scores of the G heads, then the slot's online-softmax update
#define LS_KEY_UPDATE(kx, vx, valid)                                                         \
  _Pragma("unroll") for (int g = 0; g < G; ++g) {                                            \
    float s_ = 0.f;                                                                          \
    _Pragma("unroll") for (int e = 0; e < 8; ++e) s_ = fmaf(q[g][e], kx[e], s_);             \
    _Pragma("unroll") for (int off = LPK / 2; off; off >>= 1) s_ += __shfl_xor(s_, off);     \
    s_ = (valid) ? s_ : -INFINITY;                                                           \
    const float mn_ = fmaxf(m[g], s_);                                                       \
    /* mn_ == -inf only while this slot has seen no valid key: keep everything at zero */    \
    const float corr_ = (mn_ == -INFINITY) ? 1.f : __expf(m[g] - mn_);                       \
    const float p_ = (mn_ == -INFINITY) ? 0.f : __expf(s_ - mn_);                            \
    l[g] = l[g] * corr_ + p_;                                                                \
    _Pragma("unroll") for (int e = 0; e < 8; ++e) acc[g][e] = acc[g][e] * corr_ + p_ * vx[e]; \
    m[g] = mn_;                                                                              \
  }

  // the new row first (wave 0): rotate k, round both to bf16, append to the cache, attend to
  // it.  Done before the cache stream so that the rotation table is dead inside the loop.
  if (wave == 0) {
    const bf16x8 kn = *reinterpret_cast<const bf16x8*>(row + (size_t)(hq + kh) * HD + dl * 8);
    const bf16x8 vn = *reinterpret_cast<const bf16x8*>(row + (size_t)(hq + hkv + kh) * HD + dl * 8);
    bf16x8 kr;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float u0 = (float)kn[2 * i], u1 = (float)kn[2 * i + 1];
      kr[2 * i] = (bf16)(u0 * rot[i].x - u1 * rot[i].y);
      kr[2 * i + 1] = (bf16)(u0 * rot[i].y + u1 * rot[i].x);
    }
    if (slot == 0) {
      *reinterpret_cast<bf16x8*>(kb + (size_t)pos * HD + dl * 8) = kr;
      *reinterpret_cast<bf16x8*>(vb + (size_t)pos * HD + dl * 8) = vn;
    }
    float kx[8], vx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { kx[e] = (float)kr[e]; vx[e] = (float)vn[e]; }
    const bool valid = slot == 0;
    LS_KEY_UPDATE(kx, vx, valid)
  }
  // the cache is read once per step: non-temporal loads.  The cache stream is software pipelined: the loads of the next group of U*KPI keys are
  // in flight while the current group is folded into the softmax state; a load whose keys
  // all lie past the wave's range is not issued at all
#define LS_LOAD_GROUP(buf, j0_)                                                               \
  _Pragma("unroll") for (int u = 0; u < U; ++u) {                                             \
    if ((j0_) + u * KPI < k_end) {                                                            \
      const int key_ = min((j0_) + u * KPI + slot, ctx - 1); /* clamped: a valid cache row */ \
      kf[buf][u] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(kb + (size_t)key_ * HD + dl * 8)); \
      vf[buf][u] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(vb + (size_t)key_ * HD + dl * 8)); \
    }                                                                                         \
  }
#define LS_FOLD_GROUP(buf, j0_)                                                               \
  _Pragma("unroll") for (int u = 0; u < U; ++u) {                                             \
    if ((j0_) + u * KPI < k_end) {                                                            \
      const bool valid = ((j0_) + u * KPI + slot) < k_end;                                    \
      float kx[8], vx[8];                                                                     \
      _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                         \
        kx[e] = (float)kf[buf][u][e];                                                         \
        vx[e] = (float)vf[buf][u][e];                                                         \
      }                                                                                       \
      LS_KEY_UPDATE(kx, vx, valid)                                                            \
    }                                                                                         \
  }
  {
    constexpr int STEP = KPI * U;
    bf16x8 kf[2][U], vf[2][U];
    LS_LOAD_GROUP(0, k_begin)
    for (int j0 = k_begin; j0 < k_end; j0 += 2 * STEP) {
      LS_LOAD_GROUP(1, j0 + STEP)
      LS_FOLD_GROUP(0, j0)
      LS_LOAD_GROUP(0, j0 + 2 * STEP)
      LS_FOLD_GROUP(1, j0 + STEP)
    }
  }
#undef LS_LOAD_GROUP
#undef LS_FOLD_GROUP

#undef LS_KEY_UPDATE

  // merge the key slots of the wave (lanes that hold the same dimensions)
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float mw = m[g];
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
    const float w = (m[g] == -INFINITY) ? 0.f : __expf(m[g] - mw);
    float lw = l[g] * w;
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) lw += __shfl_xor(lw, off);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float a = acc[g][e] * w;
#pragma unroll
      for (int off = LPK; off < 64; off <<= 1) a += __shfl_xor(a, off);
      acc[g][e] = a;
    }
    if (lane < LPK) {
      if (dl == 0) { sm_m[wave][g] = mw; sm_l[wave][g] = lw; }
#pragma unroll
      for (int e = 0; e < 8; ++e) sm_acc[wave][g][dl * 8 + e] = acc[g][e];
    }
  }
  __syncthreads();

  // merge the waves in wave order and write the output row
  for (int i = threadIdx.x; i < G * HD; i += NW * 64) {
    const int g = i / HD, d = i % HD;
    float mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mm = fmaxf(mm, sm_m[w][g]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float wt = (sm_m[w][g] == -INFINITY) ? 0.f : __expf(sm_m[w][g] - mm);
      num += sm_acc[w][g][d] * wt;
      den += sm_l[w][g] * wt;
    }
    out[(size_t)r * (hkv * G * HD) + (size_t)(kh * G + g) * HD + d] = (bf16)(num / den);
  }
}

template <int HD, int G>
void launch_g(const void* qkv, int qkv_stride, const float* cs, void* kc, void* vc, const int32_t* row_seq,
              const int32_t* row_pos, int rows, int hkv, int max_seq, void* out, hipStream_t st) {
  dim3 grid(rows, hkv);
  k_attn_decode<HD, G><<<grid, waves_for(G) * 64, 0, st>>>((const bf16*)qkv, qkv_stride, (const float2*)cs, (bf16*)kc, (bf16*)vc,
                                                  row_seq, row_pos, hkv * G, hkv, max_seq, (bf16*)out);
}

template <int HD>
bool launch_hd(int g, const void* qkv, int qkv_stride, const float* cs, void* kc, void* vc, const int32_t* row_seq,
               const int32_t* row_pos, int rows, int hkv, int max_seq, void* out, hipStream_t st) {
  switch (g) {
    case 1: launch_g<HD, 1>(qkv, qkv_stride, cs, kc, vc, row_seq, row_pos, rows, hkv, max_seq, out, st); return true;
    case 2: launch_g<HD, 2>(qkv, qkv_stride, cs, kc, vc, row_seq, row_pos, rows, hkv, max_seq, out, st); return true;
    case 4: launch_g<HD, 4>(qkv, qkv_stride, cs, kc, vc, row_seq, row_pos, rows, hkv, max_seq, out, st); return true;
    case 8: launch_g<HD, 8>(qkv, qkv_stride, cs, kc, vc, row_seq, row_pos, rows, hkv, max_seq, out, st); return true;
  }
  return false;
}

}  // namespace

bool attn_decode_supported(int hq, int hkv, int hd) {
  const int g = hq / hkv;
  return (hd == 128 || hd == 64) && (g == 1 || g == 2 || g == 4 || g == 8);
}

void launch_attn_decode(const void* qkv, int qkv_stride, const float* cs_table, void* kc, void* vc,
                        const int32_t* row_seq, const int32_t* row_pos, int rows, int hq, int hkv, int hd,
                        int max_seq, void* out, hipStream_t st) {
  if (rows <= 0) return;
  const int g = hq / hkv;
  if (hd == 128) launch_hd<128>(g, qkv, qkv_stride, cs_table, kc, vc, row_seq, row_pos, rows, hkv, max_seq, out, st);
  else launch_hd<64>(g, qkv, qkv_stride, cs_table, kc, vc, row_seq, row_pos, rows, hkv, max_seq, out, st);
}

}  // namespace ls
