// bf16 decode attention for grouped-query models (head_dim 128, G = Hq/Hkv query heads per KV
// head, 2 <= G <= 16), fused with RoPE and the KV-cache append of the new row.
//
// One query row per sequence, but G heads share every cached key and value, so both products
// are small matrix products and run on the matrix cores; the vector ALUs only do the softmax.
// The kernel stays bound by streaming the cache out of HBM once per step.
//
//   * One workgroup per (sequence, kv head, chunk of the context); its NW wavefronts split the
//     chunk's 32-key tiles into contiguous runs (split-KV inside the workgroup, merged in wave
//     order).  A sequence that is one chunk is one workgroup, which writes the output row; a
//     sequence of several chunks is several workgroups, each of which leaves its running
//     maximum, its sum and its un-normalised output in a scratch buffer, and a small second
//     kernel adds them up in chunk order (a fixed order: the result does not depend on timing).
//     Measured at the 70B shape (64 ragged contexts of 128..2300 keys, 8 kv heads = 512
//     workgroups): chunks of 512 keys make the kernel 24 % slower, 1024 keys 11 %, and two
//     chunks per sequence with a merge kernel 12 us per layer slower than one -- a workgroup's
//     start (query rotation, first tile) and end (merge through LDS, partial result) cost
//     several microseconds, more than the ragged batch loses by waiting for its longest
//     sequence.  So contexts are cut only where sequences x kv heads alone would leave the
//     chip idle, or beyond 8192 keys (see the constants below).
//   * A tile (32 keys x 256 bytes of K, the same of V) is fetched with sixteen 16-byte-per-lane
//     non-temporal loads, a quarter-wave per cache row (whole rows, 1 KB per instruction), and
//     goes through a wave-private LDS area (written lane-linear; the 16-byte chunks of a row
//     are XOR-swizzled on the way in so that the operand reads below hit distinct banks).
//     The loads of the next tile are in flight while the current one is processed.
//   * S^T[key][head] = K Q^T: v_mfma_f32_16x16x32_bf16 with 16 keys as the A rows and the
//     (rotated, bf16) query heads as the B columns, padded with zero heads up to 16.  A lane of
//     the result holds head = lane%16 and keys 4*(lane/16)+r of the 16: one head per lane, so
//     the running maximum and sum are per-lane values plus an exchange with lanes +-16, +-32.
//   * O^T[d][head] += V^T P^T: the eight probabilities a lane holds for a tile are exactly a
//     B operand whose k index runs over keys {4g..4g+3, 16+4g..16+4g+3} (g = lane/16); the V^T
//     operand for row d comes out of two transposing LDS reads (ds_read_b64_tr_b16) of the
//     row-major V tile: the 16 lanes of group g address a block of 4 keys x 16 dims (lane j:
//     key j/4, dims 4(j%4)..+3) and lane j receives the four keys' values at dim j.
//   * The new row: its key is rotated and rounded to bf16, appended to the cache together
//     with the value, and patched into the LDS tile that covers position `pos`, so it takes
//     the same path as every cached key.  Cache rows past `pos` are never used: keys are
//     masked before the exponential and their values are zeroed on the way into LDS.
#include <algorithm>

#include "kernels.hpp"
#include "device_util.hpp"

namespace ls {

namespace {

constexpr int HD = 128;
constexpr int TK = 32;                   // keys per tile
constexpr int TILE_BYTES = TK * HD * 2;  // 8 KB of K, 8 KB of V
// Chunking of long contexts.  One workgroup per (sequence, kv head) is the cheapest form: a
// chunk's start (tables, query rotation, first tile) and end (partial result, merge kernel)
// cost several microseconds.  Contexts are cut into chunks only to put WG_TARGET workgroups on
// the chip when sequences x kv heads are fewer, or to keep a workgroup below TPC_MAX tiles;
// never into chunks shorter than TPC_MIN tiles.
constexpr int WG_TARGET = 512;           // two workgroups per CU
constexpr int TPC_MAX = 256;             // 8192 keys
constexpr int TPC_MIN = 16;              // 512 keys
constexpr int PART_HDR = 32;             // floats in front of a partial result: 16 maxima, 16 sums

template <int NW>
__global__ void __launch_bounds__(NW * 64)
k_attn_decode_gqa(const bf16* __restrict__ qkv, int qkv_stride, const float2* __restrict__ cs,
                  bf16* __restrict__ kc, bf16* __restrict__ vc, const int32_t* __restrict__ row_seq,
                  const int32_t* __restrict__ row_pos, int hq, int hkv, int G, int max_seq, bf16* __restrict__ out,
                  float* __restrict__ part, int nchunk, int tpc) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int r = blockIdx.x, kh = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pos = row_pos[r];
  if (pos < 0) return;  // a sequence with no room left: whole workgroup leaves together
  if ((int)blockIdx.z * tpc * TK > pos) return;  // this chunk lies beyond the sequence's context
  const int seq = row_seq[r];
  const int lr = lane & 15, lg = lane >> 4;
  bf16* kb = kc + ((size_t)seq * hkv + kh) * max_seq * HD;
  bf16* vb = vc + ((size_t)seq * hkv + kh) * max_seq * HD;
  const bf16* row = qkv + (size_t)r * qkv_stride;
  unsigned char* ks = smem + wave * (2 * TILE_BYTES);
  unsigned char* vs = ks + TILE_BYTES;

  // tiles of this workgroup's chunk of the ceil((pos+1)/32) tiles, and of this wave: a contiguous run
  const int ntile = (pos + TK) / TK;
  const int t_lo = blockIdx.z * tpc;
  // the last chunk takes whatever is left, should the caller have understated the longest context
  const int t_hi = (int)blockIdx.z == nchunk - 1 ? ntile : min(t_lo + tpc, ntile);
  const int per = (t_hi - t_lo + NW - 1) / NW;
  const int t_begin = min(t_lo + wave * per, t_hi), t_end = min(t_begin + per, t_hi);

  // per-lane load coordinates inside a tile: instruction i fetches key 4i + lg; the lane
  // lands in physical chunk lr and therefore fetches the logical chunk that belongs there
  int kchunk[8], vchunk[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int kl = 4 * i + lg;
    kchunk[i] = lr ^ (kl & 15);
    vchunk[i] = lr ^ ((kl & 7) << 1);
  }
  u32x4 kreg[8], vreg[8];
#define LS_LOAD_TILE(t)                                                                                  \
  _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                        \
    const int key_ = min((t) * TK + 4 * i + lg, max(pos - 1, 0)); /* a row the cache already holds */    \
    kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + (size_t)key_ * HD + kchunk[i] * 8)); \
    vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vb + (size_t)key_ * HD + vchunk[i] * 8)); \
  }

  f32x4 o[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;                       // l_run: this lane group's share of the sum
  const float c = 1.4426950408889634f / sqrtf((float)HD);      // scores are kept in log2 units

  if (t_begin < t_end) LS_LOAD_TILE(t_begin)  // on its way while the query operand is prepared

  // query operand: head lr (zero beyond G), dims kk*32 + 8*lg .. +7, rotated at `pos`
  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const int d0 = kk * 32 + lg * 8;
    bf16x8 qv;
#pragma unroll
    for (int e = 0; e < 8; ++e) qv[e] = (bf16)0.f;
    if (lr < G) {
      const bf16x8 raw = *reinterpret_cast<const bf16x8*>(row + (size_t)(kh * G + lr) * HD + d0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float2 t = cs[(size_t)pos * (HD / 2) + d0 / 2 + i];
        const float u0 = (float)raw[2 * i], u1 = (float)raw[2 * i + 1];
        qv[2 * i] = (bf16)(u0 * t.x - u1 * t.y);
        qv[2 * i + 1] = (bf16)(u0 * t.y + u1 * t.x);
      }
    }
    qf[kk] = qv;
  }

  for (int t = t_begin; t < t_end; ++t) {
    const int key0 = t * TK;
    // registers -> LDS; values of keys past `pos` are zeroed (their probabilities are zero, but
    // 0 * garbage must stay 0)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool live = key0 + 4 * i + lg <= pos;
      *reinterpret_cast<u32x4*>(ks + i * 1024 + lane * 16) = kreg[i];
      *reinterpret_cast<u32x4*>(vs + i * 1024 + lane * 16) = live ? vreg[i] : u32x4{0u, 0u, 0u, 0u};
    }
    // the new row, if this tile covers it: lanes 0..15 own one 16-byte chunk each
    if (pos >= key0 && pos < key0 + TK && lane < 16) {
      const int kl = pos - key0;
      const bf16x8 kn = *reinterpret_cast<const bf16x8*>(row + (size_t)(hq + kh) * HD + lane * 8);
      const bf16x8 vn = *reinterpret_cast<const bf16x8*>(row + (size_t)(hq + hkv + kh) * HD + lane * 8);
      bf16x8 kr;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float2 tt = cs[(size_t)pos * (HD / 2) + lane * 4 + i];
        const float u0 = (float)kn[2 * i], u1 = (float)kn[2 * i + 1];
        kr[2 * i] = (bf16)(u0 * tt.x - u1 * tt.y);
        kr[2 * i + 1] = (bf16)(u0 * tt.y + u1 * tt.x);
      }
      *reinterpret_cast<bf16x8*>(ks + kl * 256 + ((lane ^ (kl & 15)) << 4)) = kr;
      *reinterpret_cast<bf16x8*>(vs + kl * 256 + ((lane ^ ((kl & 7) << 1)) << 4)) = vn;
      *reinterpret_cast<bf16x8*>(kb + (size_t)pos * HD + lane * 8) = kr;
      *reinterpret_cast<bf16x8*>(vb + (size_t)pos * HD + lane * 8) = vn;
    }
    if (t + 1 < t_end) LS_LOAD_TILE(t + 1)

    // ---- S^T = K Q^T for the two 16-key halves
    f32x4 s[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int kl = h * 16 + lr;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks + kl * 256 + (((kk * 4 + lg) ^ lr) << 4));
        s[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[kk], s[h], 0, 0, 0);
      }
    }
    // ---- scale, mask, online softmax for this lane's head
    float mx = -INFINITY;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int key = key0 + h * 16 + 4 * lg + e;
        const float v = key <= pos ? s[h][e] * c : -INFINITY;
        s[h][e] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);  // finite: every tile holds at least one key <= pos
    const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
    float psum = 0.f;
    bf16x8 pf;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float p = __builtin_amdgcn_exp2f(s[h][e] - m_new);
        psum += p;
        pf[h * 4 + e] = (bf16)p;
      }
    l_run = l_run * corr + psum;
    m_run = m_new;
    // ---- O^T = O^T * corr + V^T P^T
    // transposing reads: group lg hands in keys 4 lg + j/4 (and 16 more for the second half),
    // dims 16 dt + 4 (j%4); the chunk swizzle (key & 7) << 1 spreads the 4 keys x 32 bytes of
    // the four groups over all banks twice
    {
      typedef short s16x4 __attribute__((ext_vector_type(4)));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
      const int k0 = 4 * lg + (lr >> 2), k1 = k0 + 16;
      const int sw0 = (k0 & 7) << 1, sw1 = (k1 & 7) << 1;
      const int sub = (lr & 1) * 8;  // dims 4 (j%4): chunk (j%4)/2 of the 16 dims, half (j%4)&1
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const int ch = dt * 2 + ((lr & 3) >> 1);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vs + k0 * 256 + ((ch ^ sw0) << 4) + sub));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vs + k1 * 256 + ((ch ^ sw1) << 4) + sub));
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[dt][e] *= corr;
        o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pf, o[dt], 0, 0, 0);
      }
    }
  }
#undef LS_LOAD_TILE

  // ---- merge: the lane groups of a wave (sum only; the maximum is already common), then the
  // waves through LDS in wave order
  float l_wave = l_run + __shfl_xor(l_run, 16);
  l_wave += __shfl_xor(l_wave, 32);
  __syncthreads();  // every wave is done with its tile area
  float* sm_m = reinterpret_cast<float*>(smem);             // [NW][16]
  float* sm_l = sm_m + NW * 16;                              // [NW][16]
  float* sm_o = sm_l + NW * 16;                              // [NW][16 heads][128]
  if (lg == 0) { sm_m[wave * 16 + lr] = m_run; sm_l[wave * 16 + lr] = l_wave; }
#pragma unroll
  for (int dt = 0; dt < 8; ++dt)
    *reinterpret_cast<f32x4*>(sm_o + ((wave * 16 + lr) * HD + dt * 16 + 4 * lg)) = o[dt];
  __syncthreads();
  const bool whole = ntile <= tpc || nchunk == 1;  // the sequence is this one chunk: write its output row
  float* pp = part + (((size_t)r * hkv + kh) * nchunk + blockIdx.z) * (PART_HDR + (size_t)G * HD);
  for (int i = threadIdx.x; i < G * HD; i += NW * 64) {
    const int g = i / HD, d = i % HD;
    float mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mm = fmaxf(mm, sm_m[w * 16 + g]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float mw = sm_m[w * 16 + g];
      const float wt = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mm);
      num += sm_o[(w * 16 + g) * HD + d] * wt;
      den += sm_l[w * 16 + g] * wt;
    }
    if (whole) {
      out[(size_t)r * ((size_t)hq * HD) + (size_t)(kh * G + g) * HD + d] = (bf16)(num / den);
    } else {
      pp[PART_HDR + i] = num;
      if (d == 0) { pp[g] = mm; pp[16 + g] = den; }
    }
  }
}

// Second pass for sequences longer than one chunk: the chunks' partial results in chunk order.
__global__ void __launch_bounds__(256)
k_attn_gqa_merge(const float* __restrict__ part, const int32_t* __restrict__ row_pos, int hq, int hkv, int G, int nchunk,
                 int tpc, bf16* __restrict__ out) {
  const int r = blockIdx.x, kh = blockIdx.y;
  const int pos = row_pos[r];
  if (pos < 0) return;
  const int ntile = (pos + TK) / TK;
  if (ntile <= tpc) return;  // the first pass wrote this row
  const int nch = min((ntile + tpc - 1) / tpc, nchunk);
  const size_t stride = PART_HDR + (size_t)G * HD;
  const float* p0 = part + ((size_t)r * hkv + kh) * nchunk * stride;
  for (int i = threadIdx.x; i < G * HD; i += 256) {
    const int g = i / HD, d = i % HD;
    float mm = -INFINITY;
    for (int c = 0; c < nch; ++c) mm = fmaxf(mm, p0[c * stride + g]);
    float num = 0.f, den = 0.f;
    for (int c = 0; c < nch; ++c) {
      const float wt = __builtin_amdgcn_exp2f(p0[c * stride + g] - mm);  // every chunk holds a visible key: finite
      num += p0[c * stride + PART_HDR + i] * wt;
      den += p0[c * stride + 16 + g] * wt;
    }
    out[(size_t)r * ((size_t)hq * HD) + (size_t)(kh * G + g) * HD + d] = (bf16)(num / den);
  }
}

template <int NW>
void launch_nw(const void* qkv, int qkv_stride, const float* cs, void* kc, void* vc, const int32_t* row_seq,
               const int32_t* row_pos, int rows, int hq, int hkv, int max_seq, void* out, hipStream_t st, float* part,
               int nchunk, int tpc) {
  constexpr int SMEM = NW * 2 * TILE_BYTES;  // >= the merge area: NW * (32 + 16*128) floats
  static std::atomic<uint64_t> lds_allowed{0};
  allow_dynamic_lds((const void*)k_attn_decode_gqa<NW>, SMEM, lds_allowed);
  dim3 grid(rows, hkv, nchunk);
  k_attn_decode_gqa<NW><<<grid, NW * 64, SMEM, st>>>((const bf16*)qkv, qkv_stride, (const float2*)cs, (bf16*)kc,
                                                     (bf16*)vc, row_seq, row_pos, hq, hkv, hq / hkv, max_seq, (bf16*)out,
                                                     part, nchunk, tpc);
  if (nchunk > 1)
    k_attn_gqa_merge<<<dim3(rows, hkv), 256, 0, st>>>(part, row_pos, hq, hkv, hq / hkv, nchunk, tpc, (bf16*)out);
}

}  // namespace

bool attn_decode_gqa_supported(int hq, int hkv, int hd) {
  const int g = hkv > 0 ? hq / hkv : 0;
  return hd == HD && hkv > 0 && hq % hkv == 0 && g >= 2 && g <= 16;
}

#ifndef LS_ATTN_GQA_NW
#define LS_ATTN_GQA_NW 4
#endif
namespace {
// chunks per sequence for a launch of `rows` sequences whose longest context has `tiles` tiles
int gqa_chunks(int rows, int hkv, int tiles) {
  const int base = rows * hkv;
  const int want = (WG_TARGET + base - 1) / base;
  const int by_len = (tiles + TPC_MAX - 1) / TPC_MAX;
  const int most = (tiles + TPC_MIN - 1) / TPC_MIN;
  return std::max(1, std::min(std::max(want, by_len), most));
}
size_t gqa_part_bytes(int rows, int hq, int hkv, int nchunk) {
  return (size_t)rows * hkv * nchunk * (PART_HDR + (size_t)(hq / hkv) * HD) * sizeof(float);
}
}  // namespace

// An upper bound for every launch of at most `rows` sequences and `max_keys` keys: fewer rows
// mean more chunks per sequence, but rows * hkv * chunks stays below WG_TARGET + rows * hkv
// unless the length cap decides, which adds rows * hkv * chunks-by-length.
size_t attn_decode_gqa_scratch_bytes(int rows, int hq, int hkv, int max_keys) {
  if (!attn_decode_gqa_supported(hq, hkv, HD)) return 0;
  const int tiles = (std::max(max_keys, 1) + TK - 1) / TK;
  if (tiles <= TPC_MIN) return 0;
  const int by_len = (tiles + TPC_MAX - 1) / TPC_MAX;
  const size_t slots = (size_t)WG_TARGET + (size_t)rows * hkv * (1 + by_len);
  return slots * (PART_HDR + (size_t)(hq / hkv) * HD) * sizeof(float);
}

void launch_attn_decode_gqa(const void* qkv, int qkv_stride, const float* cs_table, void* kc, void* vc,
                            const int32_t* row_seq, const int32_t* row_pos, int rows, int hq, int hkv, int max_seq,
                            void* out, hipStream_t st, int max_keys, float* scratch, size_t scratch_bytes) {
  if (rows <= 0) return;
  // chunks up to the longest context the caller vouches for; without scratch for their
  // partial results every sequence stays one workgroup (one chunk as long as the cache)
  const int tiles = (min(max(max_keys, 1), max_seq) + TK - 1) / TK;
  int nchunk = gqa_chunks(rows, hkv, tiles);
  int tpc = (tiles + nchunk - 1) / nchunk;
  nchunk = (tiles + tpc - 1) / tpc;
  if (nchunk > 1 && (!scratch || gqa_part_bytes(rows, hq, hkv, nchunk) > scratch_bytes)) nchunk = 1;
  if (nchunk == 1) tpc = (max_seq + TK - 1) / TK;
  launch_nw<LS_ATTN_GQA_NW>(qkv, qkv_stride, cs_table, kc, vc, row_seq, row_pos, rows, hq, hkv, max_seq, out, st, scratch,
                            nchunk, tpc);
}

}  // namespace ls
