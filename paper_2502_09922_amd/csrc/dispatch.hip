// Shape-based choice between the kernels of one operator.  fp32 always takes the generic
// kernels; bf16 takes an MFMA kernel wherever its shape constraints hold.
#include "kernels.hpp"

namespace ls {

bool gemm_decode_fusable(int M, int N, int K) { return gemm_skinny_supported(M, N, K); }

size_t gemm_scratch_bytes(int rows, size_t cols) {
  const size_t r = rows < 64 ? rows : 64;
  return 8 * r * cols * sizeof(float);  // up to 8 K splits
}

void launch_gemm(uint32_t dt, Epilogue epi, const void* A, const void* W, int M, int N, int K, void* out,
                 float* resid, hipStream_t st, const GemmScratch* scratch, const SkinnyFusion* fusion) {
  if (dt == BF16 && M <= 64) {
    // 17..64 rows: the wide kernel, if its shape constraints hold and the scratch is large enough
    if (M > 16 && scratch && scratch->splitk && gemm_wide_supported(M, N, K) &&
        gemm_wide_workspace_bytes(M, N, K, epi == EPI_SWIGLU) <= scratch->bytes) {
      launch_gemm_wide(epi, A, W, M, N, K, out, resid, scratch->splitk, st, fusion);
      return;
    }
    if (gemm_skinny_supported(M, N, K)) {
      launch_gemm_skinny(epi, A, W, M, N, K, out, resid, 0, st, fusion);
      return;
    }
  }
  if (dt == BF16 && M > 64 && gemm_mfma_supported(M, N, K)) {
    launch_gemm_mfma(epi, A, W, M, N, K, out, resid, st);
    return;
  }
  launch_gemm_generic(dt, epi, A, W, M, N, K, out, resid, st);
}

void launch_attention_block(uint32_t dt, const int32_t* cu_seqlens, int batch, int max_len, void* qkv,
                            const float* cs_table, void* kcache, void* vcache, const int32_t* row_seq,
                            const int32_t* row_pos, int rows, int hq, int hkv, int hd, int max_seq, void* out,
                            hipStream_t st, float* attn_scratch, size_t attn_scratch_bytes, bool rope_done) {
  const bool decode = cu_seqlens == nullptr;
  const int qkv_stride = (hq + 2 * hkv) * hd;
  if (dt == BF16 && decode && attn_decode_gqa_supported(hq, hkv, hd)) {
    launch_attn_decode_gqa(qkv, qkv_stride, cs_table, kcache, vcache, row_seq, row_pos, rows, hq, hkv, max_seq, out, st,
                           max_len, attn_scratch, attn_scratch_bytes);
    return;
  }
  if (dt == BF16 && decode && attn_decode_supported(hq, hkv, hd)) {
    launch_attn_decode(qkv, qkv_stride, cs_table, kcache, vcache, row_seq, row_pos, rows, hq, hkv, hd, max_seq, out, st);
    return;
  }
  if (!rope_done) launch_rope_append(dt, qkv, cs_table, row_seq, row_pos, rows, hq, hkv, hd, max_seq, kcache, vcache, st);
  if (dt == BF16 && !decode && attn_prefill_supported(hq, hkv, hd)) {
    launch_attn_prefill(qkv, qkv_stride, kcache, vcache, cu_seqlens, batch, max_len, hq, hkv, hd, max_seq, out, st);
    return;
  }
  launch_attention_generic(dt, qkv, qkv_stride, kcache, vcache, row_seq, row_pos, rows, hq, hkv, hd, max_seq, out, st);
}

}  // namespace ls
