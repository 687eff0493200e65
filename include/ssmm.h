/*
 * ssmm.h -- C ABI of the MI355X (gfx950) sparse-sparse MoE expert-FFN library.
 *
 * The library implements the hot path of "Samoyeds" (arxiv 2503.10725): expert
 * weights pruned to the dual-side structured format (vector-wise N-of-M Sub-Rows
 * stacked on 2:4, section 4.1) and stored as values + metadata + indices; the
 * activations sparse by routing (selection array SEL, section 4.1); one fused
 * sparse-sparse matrix multiplication per expert linear (Algorithm 1,
 * sections 4.2-4.5).
 *
 * Conventions for every entry point
 *   - plain C, no exceptions; the return value is 0 (SSMM_OK) or a negative
 *     ssmm_status; ssmm_strerror() names it.
 *   - every data pointer is a DEVICE pointer owned by the caller; the library
 *     allocates and frees nothing; scratch comes from a caller workspace whose
 *     size is queried beforehand.  Size out-parameters (size_t*) are HOST pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it; they never synchronise.
 *   - bf16 tensors are passed as uint16_t bit patterns.
 *   - argument and shape errors are detected on the host before anything is
 *     launched (SSMM_EINVAL: null pointer or bad scalar; SSMM_ESHAPE: a size
 *     the format or the kernels do not admit; SSMM_EWORKSPACE: workspace too
 *     small; SSMM_EHIP: the HIP runtime reported a launch error; SSMM_ELIMIT: a
 *     size beyond the fixed scratch of an entry point that takes no workspace).
 *   - weight matrices are given as the transposed operand A = W^T of section
 *     4.5: `rows` output features by `K` reduction elements, row-major.
 */
#ifndef SSMM_H
#define SSMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SSMM_OK = 0,
  SSMM_EINVAL = -1,
  SSMM_ESHAPE = -2,
  SSMM_EWORKSPACE = -3,
  SSMM_EHIP = -4,
  SSMM_ELIMIT = -5
} ssmm_status;

/* The expert's activation function (the paper names none: sections 2.1, 4.5; its models use
 * SiLU, OpenMoE of section 6.2 a GELU-family gate):
 *   SILU       g * sigmoid(g)
 *   GELU_TANH  0.5 g (1 + tanh(sqrt(2/pi) (g + 0.044715 g^3)))
 *   RELU       max(g, 0) */
typedef enum {
  SSMM_ACT_SILU = 1,
  SSMM_ACT_GELU_TANH = 2,
  SSMM_ACT_RELU = 3
} ssmm_activation;

/*
 * Weight sparsity format (N, M, V) of section 4.1: blocks of M consecutive rows
 * by V consecutive reduction elements; N of the M Sub-Rows of a block are kept
 * and every kept Sub-Row is then pruned 2:4.  {1, 1, 0} means plain 2:4 (no
 * vector-wise level, no index array).  Requirements: 1 <= N <= M <= 256;
 * if N < M then V is a positive multiple of 4, K % V == 0 and rows % M == 0;
 * always K % 4 == 0.
 */
typedef struct {
  int32_t N, M, V;
} ssmm_format;

/* Text for a status code; never NULL; static storage. */
const char* ssmm_strerror(int status);

/*
 * Byte sizes of one matrix (one expert) in the encoded form of section 4.1, with
 * rc = rows*N/M compressed rows (rc = rows for plain 2:4):
 *   values  rc x K/2 bf16                 (kept elements in ascending reduction order)
 *   meta    rc x ceil(K/32) uint32        (2 bits per kept value = its position in its group
 *                                          of 4; group g of a row is the nibble at bits
 *                                          4*(g%8) of word g/8, low two bits = first kept)
 *   index   rc x K/V uint8                (row offset in [0,M) of the Sub-Row kept in that
 *                                          segment; 0 bytes for plain 2:4)
 *   tiled   the kernel-ready copy (values and metadata re-ordered into the lane order
 *           of the gfx950 sparse MFMA, the idea of the metadata packing of section 4.4;
 *           for (1,2,V) also 2 source-row bits per lane and 32 reduction elements, for
 *           the other vector-wise formats one byte per dense row and 32 reduction
 *           elements that names the stored Sub-Row); 0 if it cannot be tiled: the format
 *           must be plain 2:4, or (1,2,V) with V a multiple of 8, or (N,M,V) with M a
 *           power of two <= 32, M/N a power of two and V a multiple of 32 (then also
 *           rows % 32 == 0), with rc % 32 == 0 and K % 64 == 0.
 * Any out-pointer may be NULL.  Host function, no GPU work.
 */
int ssmm_compressed_sizes(int64_t rows, int64_t K, ssmm_format f, size_t* values_bytes,
                          size_t* meta_bytes, size_t* index_bytes, size_t* tiled_bytes);

/*
 * Prune and encode E dense matrices (section 4.1; pruning criterion: magnitude --
 * Sub-Rows ranked by the fp64 sum of squares of their V unpruned values, then the
 * two largest |v| of every group of 4; equal scores go to the lower row / lower
 * position; a NaN weight ranks like an infinity in both steps, so it is kept and stays
 * visible in the outputs).
 *   w_dense  in   bf16 [E][rows][K]
 *   values   out  bf16 [E][rc][K/2]          canonical, may be NULL together with meta/index
 *   meta     out  u32  [E][rc][ceil(K/32)]   canonical
 *   index    out  u8   [E][rc][K/V]          canonical; ignored (may be NULL) for plain 2:4
 *   tiled    out  E * tiled_bytes            kernel-ready form, may be NULL
 * Either the canonical triple or `tiled` (or both) must be given; producing
 * `tiled` without a canonical destination is allowed for plain 2:4 (a vector-wise
 * format keeps its Sub-Row choice in `index`, so the canonical triple is required).
 */
int ssmm_compress_weights(const uint16_t* w_dense, int E, int64_t rows, int64_t K, ssmm_format f,
                          uint16_t* values, uint32_t* meta, uint8_t* index, void* tiled,
                          void* stream);

/*
 * Inverse of the encoding: the pruned dense matrices, bit for bit (kept values
 * keep their bits, pruned positions are +0.0).  w_dense_out bf16 [E][rows][K].
 */
int ssmm_decompress_weights(const uint16_t* values, const uint32_t* meta, const uint8_t* index,
                            int E, int64_t rows, int64_t K, ssmm_format f, uint16_t* w_dense_out,
                            void* stream);

/*
 * Kernel-ready form back to the canonical arrays (the tiling is a bijection;
 * this is its inverse, used to verify it).
 */
int ssmm_untile_weights(const void* tiled, int E, int64_t rows, int64_t K, ssmm_format f,
                        uint16_t* values, uint32_t* meta, uint8_t* index, void* stream);

/*
 * Kernel-ready form of a gathered vector-wise format -> kernel-ready form of plain 2:4
 * of the same pruned matrices: every dense row gets its operands, pruned Sub-Rows as
 * zeros (section 4.1 read backwards for the Sub-Row level only; the 2:4 level stays
 * encoded).  M/N times the bytes, no gather in the inner loop: the form to keep
 * beside the compact one for large token counts, where the layer is bound by the MFMAs
 * and the Sub-Row level saves none (ssmm_expert_ffn otherwise expands on every call
 * into its workspace when buckets are large).
 *   tiled        in   E x tiled_bytes of (rows, K, f), device
 *   tiled_plain  out  E x tiled_bytes of (rows, K, {1,1,0}), device, 16-byte aligned
 * f must be a format with a gathered kernel-ready form ((N,M,V), M a power of two
 * <= 32, M/N a power of two >= 2 other than (1,2,V), V % 32 == 0) and (rows, K) must be
 * tileable in both forms: SSMM_ESHAPE otherwise.
 */
int ssmm_expand_tiled_weights(const void* tiled, int E, int64_t rows, int64_t K, ssmm_format f,
                              void* tiled_plain, void* stream);

/*
 * Token routing and selection arrays (sections 2.1, 3.1 and 4.1 "SEL"; shared
 * experts of section 6.2).  The paper gives no router formula; this one is
 * softmax over the E logits of a token, the `topk` largest logits (equal logits:
 * lower expert id first) in descending order, weight = softmax probability,
 * divided by the sum of the chosen ones when `renormalize` != 0.  Shared
 * experts have ids E..E+n_shared-1, weight 1, and take every token.
 * A logit of -infinity masks an expert (weight 0); a NaN logit counts as -infinity.  When a
 * token has fewer than `topk` logits above -infinity the rest of its choice goes by ascending
 * expert id, so its ids are always distinct; a token without any logit above -infinity
 * gets ids 0..topk-1 and weights that are not numbers.
 *   logits          in   f32 [T][E]
 *   topk_ids        out  i32 [T][topk]
 *   topk_w          out  f32 [T][topk]
 *   expert_offsets  out  i32 [E+n_shared+1]   exclusive scan of the per-expert token counts
 *   sel             out  i32 [P]              token id per bucket position, ascending inside
 *                                             an expert; P = T*(topk+n_shared)
 *   sel_w           out  f32 [P]              routing weight of that (token, expert) pair
 *   inv             out  i32 [T][topk+n_shared]  bucket position of every (token, slot)
 *   workspace            ssmm_route_workspace_bytes() bytes, 256-byte aligned
 * Limits: 1 <= topk <= min(E, 16); E + n_shared <= 256; T >= 0 (T = 0 only
 * writes zero offsets).
 */
size_t ssmm_route_workspace_bytes(int T, int E, int topk, int n_shared);

/*
 * The router in front of ssmm_route_bucket (section 2.1: the gate network is a linear layer
 * from the hidden state to one logit per routed expert):
 *   logits[t][e] = sum over k of x[t][k] * wr[e][k]
 * bf16 operands, fp32 accumulation in a fixed order (repeated calls return identical bits).
 *   x       in   bf16 [T][H]
 *   wr      in   bf16 [E][H]   (dense: the router is not pruned)
 *   logits  out  f32  [T][E]
 * Limits: H % 16 == 0, E <= 256 (SSMM_ESHAPE).  No workspace.
 */
int ssmm_router_logits(const uint16_t* x, int T, int H, const uint16_t* wr, int E, float* logits,
                       void* stream);
int ssmm_route_bucket(const float* logits, int T, int E, int topk, int n_shared, int renormalize,
                      int32_t* topk_ids, float* topk_w, int32_t* expert_offsets, int32_t* sel,
                      float* sel_w, int32_t* inv, void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * ssmm_route_bucket for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (without the workspace), same kernels, same outputs bit for
 * bit.  The per-chunk histograms the kernels keep between their launches live in a fixed
 * 256 KiB array inside the library, one copy per GPU, held until the process ends; the
 * call allocates and frees nothing and calls no allocating routine.
 * Limit: ceil(T / 256) * E <= 65536 (e.g. 65536 tokens with 256 experts, 262144 with 64);
 * beyond it the call returns SSMM_ELIMIT and launches nothing.  Every call on a GPU uses
 * that GPU's one array: calls that overlap on one GPU (two streams, two host threads) race
 * and must be serialised by the caller; nothing in the array needs clearing between calls.
 */
int ssmm_route_bucket_noalloc(const float* logits, int T, int E, int topk, int n_shared, int renormalize,
                              int32_t* topk_ids, float* topk_w, int32_t* expert_offsets, int32_t* sel,
                              float* sel_w, int32_t* inv, void* stream);

/*
 * The expert FFNs of one MoE layer as sparse-sparse matrix multiplications
 * (Algorithm 1; fusion of the activation and of the weighted accumulation:
 * section 4.3; compressed intermediate layout: section 4.5):
 *   for every expert e and every bucket position p of e, with t = sel[p]:
 *     h[p]  = silu(Wg_e x[t]) * (Wu_e x[t])                 (stored bf16, bucket order)
 *     o[p]  = sel_w[p] * (Wd_e h[p])
 *   y[t]    = sum over the token's slots j, in slot order, of o[inv[t][j]]
 * bf16 inputs, fp32 accumulation, bf16 output.
 *   x               in   bf16 [T][H]
 *   wg, wu          in   kernel-ready gate / up weights of the E_total experts
 *                        (rows = F, K = H), as ssmm_compress_weights wrote them
 *   wd              in   kernel-ready down weights (rows = H, K = F)
 *   expert_offsets, sel, sel_w, inv   as ssmm_route_bucket wrote them (slots = topk+n_shared)
 *   y               out  bf16 [T][H]
 *   workspace            ssmm_ffn_workspace_bytes() bytes, 256-byte aligned
 * Formats the kernels admit: those with a kernel-ready form (ssmm_compressed_sizes):
 * plain 2:4; (1,2,V)+2:4 with V a multiple of 8 (the vector-wise level halves the
 * weight bytes; the sparse MFMA spans 32 reduction elements, so both candidate rows
 * of a pair are still multiplied); (N,M,V)+2:4 such as (4,8,32) and (8,16,32)
 * (operands of the dense rows gathered from the stored Sub-Rows: weight bytes shrink
 * by N/M, the multiplications are those of plain 2:4, on slower kernels; with large
 * buckets the call first expands the weights to plain 2:4 operand order inside the
 * workspace, which ssmm_ffn_workspace_bytes() then sizes for it).
 * Shapes: H % 64 == 0, F % 64 == 0 (both are reduction lengths and row counts),
 * compressed row counts multiples of 32 (so H % 64 == 0 and F % 64 == 0 again for
 * (1,2,V)), H % V == 0 and F % V == 0; E_total <= 512 (SSMM_ESHAPE beyond).  Sums along the reduction have a fixed
 * order that depends only on the shapes and bucket sizes (the down projection splits
 * its reduction into slices whenever its tiles would not fill the chip: small buckets,
 * large buckets of few experts), so repeated calls return identical bits.
 */
size_t ssmm_ffn_workspace_bytes(int T, int H, int F, int E_total, int slots, ssmm_format f);
int ssmm_expert_ffn(const uint16_t* x, int T, int H, int F, int E_total, ssmm_format f,
                    const void* wg_tiled, const void* wu_tiled, const void* wd_tiled,
                    const int32_t* expert_offsets, const int32_t* sel, const float* sel_w,
                    const int32_t* inv, int slots, uint16_t* y, void* workspace,
                    size_t workspace_bytes, void* stream);

/*
 * Same call for callers that measure the kernels of the path (the "where time goes"
 * break-down of section 6.4): `events` is NULL or a HOST array of four hipEvent_t
 * created by the caller; they are recorded on `stream` before the gate/up product,
 * after it, after the down product and after the combine.  Nothing is synchronised;
 * the caller reads the elapsed times after it has synchronised the stream itself.
 */
int ssmm_expert_ffn_timed(const uint16_t* x, int T, int H, int F, int E_total, ssmm_format f,
                          const void* wg_tiled, const void* wu_tiled, const void* wd_tiled,
                          const int32_t* expert_offsets, const int32_t* sel, const float* sel_w,
                          const int32_t* inv, int slots, uint16_t* y, void* workspace,
                          size_t workspace_bytes, void* stream, void* const* events);

/*
 * Layer variants (the experts of section 2.1 with another activation function, and experts
 * without a gate: h[p] = act(W1_e x[t]), the form of the OpenMoE experiment of section 6.2 as
 * far as the paper describes it).  Same arguments, rules and event marks as
 * ssmm_expert_ffn_timed, plus
 *   activation   one of ssmm_activation (SSMM_EINVAL otherwise)
 *   gated        non-zero: h = act(Wg x) * (Wu x); zero: h = act(Wg x), wu_tiled is ignored
 *                and may be NULL
 * ssmm_expert_ffn(...) is this call with SSMM_ACT_SILU, gated.
 */
int ssmm_expert_ffn_variant(const uint16_t* x, int T, int H, int F, int E_total, ssmm_format f, int activation,
                            int gated, const void* wg_tiled, const void* wu_tiled, const void* wd_tiled,
                            const int32_t* expert_offsets, const int32_t* sel, const float* sel_w,
                            const int32_t* inv, int slots, uint16_t* y, void* workspace,
                            size_t workspace_bytes, void* stream, void* const* events);

/*
 * The sparse-sparse matrix multiplication on its own (section 4.1; the kernel
 * benchmarks of section 6.1 run it): C = A x B[:, SEL] with A one encoded weight
 * matrix, B given with one row per column of the paper's B (K contiguous per
 * column, the transposed packing of section 4.4), the result in the compressed
 * output layout of section 4.5 (only the selected columns, in selection order):
 *   c[j][r] = sum over k of A[r][k] * b[sel[j]][k]       (bf16 in, fp32 accumulate, bf16 out)
 *   a_tiled  in   kernel-ready form of ONE matrix (rows x K) as ssmm_compress_weights wrote it
 *   b        in   bf16 [n_b][K]; n_b * K * 2 bytes must stay below 4 GiB
 *   sel      in   i32 [n], values in [0, n_b) (not checked); NULL selects columns 0..n-1
 *   c        out  bf16 [n][rows]
 *   workspace     ssmm_matmul_workspace_bytes(rows, K, n, f) bytes, 256-byte aligned
 *                 (when rows and n give too few tiles to fill the chip the reduction
 *                 is cut into slices whose fp32 partial sums live here and are added
 *                 in a fixed order)
 * Same formats and shape rules as ssmm_expert_ffn (rows*N/M % 32 == 0, K % 64 == 0).
 */
size_t ssmm_matmul_workspace_bytes(int64_t rows, int64_t K, int n, ssmm_format f);
int ssmm_matmul(const void* a_tiled, int64_t rows, int64_t K, ssmm_format f, const uint16_t* b, int64_t n_b,
                const int32_t* sel, int n, uint16_t* c, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SSMM_H */
