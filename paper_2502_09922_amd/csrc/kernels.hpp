// Internal launcher interface between the stage runtime and the HIP kernels (gfx950).
// Every launcher only enqueues on `st`; shapes are validated by the runtime before.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ls {

enum : uint32_t { F32 = 0, BF16 = 1 };

// printf-style setter of the thread-local message behind ls_last_error()
void set_last_error(const char* fmt, ...);

// One-shot request to time the next kernel launch that goes through launch_kernel() on this
// thread: the HIP runtime stamps `start` / `stop` with that kernel's own begin and end (no
// launch gap inside the span, unlike a pair of events recorded around the launch).
struct LaunchTiming {
  hipEvent_t start = nullptr, stop = nullptr;
  bool used = false;
};
LaunchTiming& launch_timing();

// What a GEMM does with its fp32 accumulators.
enum Epilogue : int {
  EPI_STORE = 0,   // out[M,N] in dtype
  EPI_RESID = 1,   // resid[M,N] (fp32) += acc
  EPI_SWIGLU = 2,  // W is [2N,K] (gate rows then up rows); out[M,N] = silu(gate) * up, dtype
  EPI_F32 = 3      // out[M,N] fp32
};

// row_seq[r] / row_pos[r]: sequence and cache position of every row of a call.
void launch_row_index_prefill(const int32_t* cu_seqlens, int batch, int total, int32_t* row_seq,
                              int32_t* row_pos, int32_t* last_rows, hipStream_t st);
// Decode: row b is sequence b at position seq_lens[b]; -1 marks a row that has no room left.
void launch_row_index_decode(const int32_t* seq_lens, int batch, int max_seq, int32_t* row_seq,
                             int32_t* row_pos, int32_t* last_rows, hipStream_t st);
void launch_seq_lens_set(const int32_t* cu_seqlens, int batch, int32_t* seq_lens, hipStream_t st);
void launch_seq_lens_inc(int batch, int max_seq, int32_t* seq_lens, hipStream_t st);

// Decode step, fused path: row maps + seq_lens increment + fp32 residual rows + their
// storage-type copy xb (times a gain) + per-16-column sums of squares ss_part[batch][d/16], one launch.
// table != nullptr: `in` holds int32 token ids and rows are gathered from the table.
// xb = storage-type copy of the rows times gamma (the gain of the first norm; nullptr: none).
void launch_decode_prologue(uint32_t dt, const void* table, const void* in, int32_t* seq_lens, int batch, int max_seq,
                            int d, int vocab, int32_t* row_seq, int32_t* row_pos, int32_t* last_rows, float* x,
                            void* xb, float* ss_part, const void* gamma, hipStream_t st);

void launch_embed(uint32_t dt, const void* table, const int32_t* tok, float* x, int rows, int d,
                  int vocab, hipStream_t st);
void launch_load_hidden(uint32_t dt, const void* in, float* x, size_t n, hipStream_t st);
void launch_store_hidden(uint32_t dt, const float* x, void* out, size_t n, hipStream_t st);

// y[r,:] = x[map ? map[r] : r, :] / sqrt(mean(x^2) + eps) * gamma
void launch_rmsnorm(uint32_t dt, const float* x, const void* gamma, void* y, int rows, int d,
                    float eps, const int32_t* row_map, hipStream_t st);

// Scratch for GEMM kernels that split K across workgroups (fp32 partial tiles).
struct GemmScratch {
  float* splitk = nullptr;
  size_t bytes = 0;
};
struct SkinnyFusion;

// C = A[M,K] * W[N,K]^T with fp32 accumulation; A, W in dtype.  `fusion` (decode steps only)
// folds an RMSNorm into the GEMM; the caller must have checked gemm_decode_fusable().
void launch_gemm(uint32_t dt, Epilogue epi, const void* A, const void* W, int M, int N, int K,
                 void* out, float* resid, hipStream_t st, const GemmScratch* scratch = nullptr,
                 const SkinnyFusion* fusion = nullptr);
bool gemm_decode_fusable(int M, int N, int K);
// fp32 bytes of split-K scratch that cover any GEMM of up to `rows` (<= 64) rows and `cols`
// columns (count 2F for the gate-up projection)
size_t gemm_scratch_bytes(int rows, size_t cols);

void launch_gemm_generic(uint32_t dt, Epilogue epi, const void* A, const void* W, int M, int N, int K,
                         void* out, float* resid, hipStream_t st);

// bf16 MFMA kernel for many-row GEMMs (prompt pass); needs K % 64 == 0.
bool gemm_mfma_supported(int M, int N, int K);
void launch_gemm_mfma(Epilogue epi, const void* A, const void* W, int M, int N, int K, void* out, float* resid,
                      hipStream_t st);
// The QKV projection of a prompt pass with RoPE and the KV-cache append in its epilogue: rotated
// query rows go to out[M,N] (N = (hq + 2 hkv) hd, key and value columns of `out` are not
// written), rotated keys and the values go to their cache rows (row_seq[m], row_pos[m]; rows
// with row_pos < 0 are skipped).  head_dim 64 or 128.
struct RopeAppend {
  const float* cs = nullptr;        // cos/sin table [max_seq][hd/2][2]
  const int32_t* row_seq = nullptr;
  const int32_t* row_pos = nullptr;
  int hq = 0, hkv = 0, hd = 0, max_seq = 0;
  __bf16* kc = nullptr;
  __bf16* vc = nullptr;
};
bool gemm_mfma_rope_supported(int M, int N, int K, int hq, int hkv, int hd);
void launch_gemm_mfma_rope(const void* A, const void* W, int M, int N, int K, void* out, const RopeAppend& rope,
                           hipStream_t st);

// bf16 weight-streaming kernel for decode steps (M <= 64); needs N % 16 == 0, K % 128 == 0.
// ks = wavefronts that split K inside a workgroup (4, 8, 16), 0 = chosen from the shape.
// Optional RMSNorm fusion of the decode step (all pointers device memory).  The gain of a
// norm is applied by whoever PRODUCES the bf16 copy of the residual rows, the row scale by
// the GEMM that CONSUMES it:
//   xb_out != nullptr (EPI_RESID): also write xb_out[M,N] = bf16(x_new * gamma_out[n])
//     (gamma_out == nullptr: no gain) and each row's sum of squares of x_new per 16-column
//     tile to ss_out[M][N/16].
//   ss_in != nullptr (EPI_STORE / EPI_SWIGLU): X is such a copy; the accumulator is scaled
//     by 1/sqrt(sum(ss_in[row][0..n_part)) / K + eps) of its row in the epilogue.
struct SkinnyFusion {
  const float* ss_in = nullptr;
  int n_part = 0;
  float eps = 0.f;
  __bf16* xb_out = nullptr;
  float* ss_out = nullptr;
  const __bf16* gamma_out = nullptr;
};
bool gemm_skinny_supported(int M, int N, int K);
void launch_gemm_skinny(Epilogue epi, const void* X, const void* W, int M, int N, int K, void* out, float* resid,
                        int ks, hipStream_t st, const SkinnyFusion* fusion = nullptr);

// bf16 weight-streaming kernel for decode batches of 17..64 rows (K split across
// workgroups, X staged once per workgroup); needs N % 64 == 0, K % 128 == 0.
bool gemm_wide_supported(int M, int N, int K);
size_t gemm_wide_workspace_bytes(int M, int N, int K, bool glu);
void launch_gemm_wide(Epilogue epi, const void* X, const void* W, int M, int N, int K, void* out, float* resid,
                      float* splitk_ws, hipStream_t st, const SkinnyFusion* fusion);

// Rotate q (in place inside qkv) and k by the per-position cos/sin table, write k and v
// into the cache at [seq][kv head][pos].  qkv is [rows, (Hq+2Hkv)*hd].
void launch_rope_append(uint32_t dt, void* qkv, const float* cs_table, const int32_t* row_seq,
                        const int32_t* row_pos, int rows, int hq, int hkv, int hd, int max_seq,
                        void* kcache, void* vcache, hipStream_t st);

// Causal attention of every row against its sequence's cache positions 0..row_pos[r].
// q is read from qkv ([rows, qkv_stride]); out is [rows, Hq*hd].
// Attention of one layer, including RoPE and the KV-cache append of the call's rows.
// qkv [rows, (Hq+2Hkv)*hd] holds the un-rotated projections and may be rotated in place.
// Decode (cu_seqlens == nullptr): every row is the single new row of its sequence; max_len is
// then an upper bound of the keys a row attends to, and attn_scratch the buffer for the
// partial results of contexts that are split over several workgroups (may be nullptr).
// Prefill: sequence b owns rows [cu_seqlens[b], cu_seqlens[b+1]) at positions 0.., the
// longest sequence has max_len rows.  out is [rows, Hq*hd].
void launch_attention_block(uint32_t dt, const int32_t* cu_seqlens, int batch, int max_len, void* qkv,
                            const float* cs_table, void* kcache, void* vcache, const int32_t* row_seq,
                            const int32_t* row_pos, int rows, int hq, int hkv, int hd, int max_seq, void* out,
                            hipStream_t st, float* attn_scratch = nullptr, size_t attn_scratch_bytes = 0,
                            bool rope_done = false);

// bf16 split-KV decode attention fused with RoPE and the cache append; head_dim 64 or 128,
// Hq/Hkv in {1,2,4,8}.
bool attn_decode_supported(int hq, int hkv, int hd);
void launch_attn_decode(const void* qkv, int qkv_stride, const float* cs_table, void* kc, void* vc,
                        const int32_t* row_seq, const int32_t* row_pos, int rows, int hq, int hkv, int hd,
                        int max_seq, void* out, hipStream_t st);

// bf16 decode attention on the matrix cores for grouped-query models (head_dim 128,
// 2 <= Hq/Hkv <= 16), fused with RoPE and the cache append like launch_attn_decode.
bool attn_decode_gqa_supported(int hq, int hkv, int hd);
// max_keys: an upper bound of the keys any row attends to in this step (cached + the new one);
// contexts longer than 512 keys are cut into chunks that run as workgroups of their own and
// leave partial results in `scratch` (attn_decode_gqa_scratch_bytes; none: one workgroup per
// sequence and kv head whatever its length).
size_t attn_decode_gqa_scratch_bytes(int rows, int hq, int hkv, int max_keys);
void launch_attn_decode_gqa(const void* qkv, int qkv_stride, const float* cs_table, void* kc, void* vc,
                            const int32_t* row_seq, const int32_t* row_pos, int rows, int hq, int hkv, int max_seq,
                            void* out, hipStream_t st, int max_keys, float* scratch, size_t scratch_bytes);

// bf16 flash-style causal attention for the prompt pass; head_dim 64 or 128.
bool attn_prefill_supported(int hq, int hkv, int hd);
void launch_attn_prefill(const void* qkv, int qkv_stride, const void* kc, const void* vc, const int32_t* cu_seqlens,
                         int batch, int max_len, int hq, int hkv, int hd, int max_seq, void* out, hipStream_t st);

// bf16 split-KV decode attention; head_dim 64 or 128, Hq/Hkv in {1,2,4,8}.
bool attn_decode_supported(int hq, int hkv, int hd);
void launch_attn_decode(const void* qkv, int qkv_stride, const void* kc, const void* vc, const int32_t* row_seq,
                        const int32_t* row_pos, int rows, int hq, int hkv, int hd, int max_seq, void* out,
                        hipStream_t st);

void launch_attention_generic(uint32_t dt, const void* qkv, int qkv_stride, const void* kcache,
                              const void* vcache, const int32_t* row_seq, const int32_t* row_pos, int rows,
                              int hq, int hkv, int hd, int max_seq, void* out, hipStream_t st);

// tok[r] = index of the largest logit of row r, lowest index on ties.
void launch_argmax(const float* logits, int rows, int vocab, int32_t* tok, hipStream_t st);

}  // namespace ls
