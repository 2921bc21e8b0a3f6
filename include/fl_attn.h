/*
 * fl_attn.h -- C ABI of the fused attention-variant library for AMD MI355X (gfx950): the forward
 * pass of every variant, the backward pass of the variants without bias, gate and second stream, and the
 * decode step (one query per sequence over a paged key/value cache).
 *
 * One call computes, for every (b, g, h) and every query row i, without ever writing the
 * [Sq, Sk] score matrix to device memory:
 *
 *     s_ij   = scale * <q_i, k_j>                                     (paper Eq. 3)
 *     s_ij   = score_mod(s_ij)                 soft-cap / ALiBi       (paper Eq. 4)
 *     s_ij  += bias_0[b,g,h,i,j] + bias_1[b,g,h,i,j]                  (Evoformer biases, Sec. 4.1)
 *     s_ij   = -inf where masked               causal / window / prefix / document
 *                                              (attention listing; sliding-window listings)
 *     P_ij   = softmax over j, computed with the online recurrence    (Eq. 2, Alg. 2, Sec. 3.4)
 *     o_i    = sum_j P_ij v_j                                         (Eq. 3)
 *     differential:  o_i = o_i(q,k) - lambda_h * o_i(q2,k2), same v   (differential listing)
 *     epilogue:      RMSNorm over the Dv channels, then * sigmoid(gate)
 *     lse_i  = m_i + ln(l_i)   (m_i, l_i: post-condition of Alg. 1 / Alg. 2)
 *
 * Fixed order of the score pipeline when several parts are enabled:
 *     scale -> soft-cap -> ALiBi -> + biases -> mask.
 *
 * All tensor pointers are DEVICE pointers owned by the caller.  The library never allocates,
 * frees or keeps device memory; work is enqueued on the caller's stream and the call returns
 * without synchronising.  Every validation failure returns before anything is launched and
 * leaves the outputs untouched.  There is no CPU fallback and no generic slow path: a bf16
 * descriptor without a compiled specialisation is instantiated from the same kernel templates on
 * its first use (hipRTC, a few seconds, once per process); head dims outside {32, 64, 128} are
 * FL_ERR_UNSUPPORTED.
 */
#ifndef FL_ATTN_H
#define FL_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FL_OK = 0,
  FL_ERR_NULL = 1,         /* a required pointer is NULL                                   */
  FL_ERR_DTYPE = 2,        /* dtype combination not supported                              */
  FL_ERR_SHAPE = 3,        /* sizes inconsistent between tensors                           */
  FL_ERR_STRIDE = 4,       /* innermost stride != 1, or a negative / forbidden-zero stride */
  FL_ERR_ALIGN = 5,        /* base pointer or row stride not 16-byte aligned               */
  FL_ERR_UNSUPPORTED = 6,  /* no compiled specialisation for this descriptor / head dim    */
  FL_ERR_AUX_MISSING = 7,  /* descriptor needs an aux tensor that was not given            */
  FL_ERR_WORKSPACE = 8,    /* workspace NULL or smaller than fl_attn_fwd_workspace_size    */
  FL_ERR_LAUNCH = 9,       /* the HIP runtime refused a launch (see fl_last_error_detail)  */
  FL_ERR_DESC = 10         /* descriptor fields contradict each other / bad struct_size    */
} fl_status;

typedef enum { FL_BF16 = 1, FL_F32 = 2, FL_I32 = 3 } fl_dtype;

/* A strided view with logical dims [B, G, H, S, D].
 *   G is an extra independent row axis: 1 for ordinary attention, the MSA-sequence axis for
 *   Evoformer row-wise attention.  Strides are in ELEMENTS.  stride[4] must be 1.
 *   For q/k/v/out/gate all strides are >= 0 and every row (last axis) starts 16-byte aligned.
 *   Bias tensors have logical dims [B, G, H, Sq, Sk]; a stride of 0 broadcasts that axis.   */
typedef struct {
  void*   ptr;
  int32_t dtype;           /* fl_dtype */
  int32_t reserved;
  int64_t size[5];
  int64_t stride[5];
} fl_tensor;

/* score_mod (paper Eq. 4): elementwise old score -> new score, on the SCALED score. */
enum { FL_MOD_NONE = 0, FL_MOD_ALIBI = 1, FL_MOD_SOFTCAP = 2 };

/* mask bits (True = masked, combined by OR), i = query index, j = key index:
 * (with q_offset != 0 read i as the query's position i + q_offset in the three positional masks)
 *   CAUSAL  masked iff j > i                                   (attention listing + causal)
 *   WINDOW  masked iff j > i or i - j > window                 (sliding-window listings);
 *           implies CAUSAL, so window + 1 keys are visible including j = i
 *   PREFIX  masked iff j > i and j >= prefix_len               (PrefixLM, Sec. 4.1); excludes
 *           CAUSAL and WINDOW
 *   DOC     masked iff q_doc_ids[b,i] != kv_doc_ids[b,j]       (Document mask, Sec. 4.1)      */
enum { FL_MASK_CAUSAL = 1, FL_MASK_WINDOW = 2, FL_MASK_DOC = 4, FL_MASK_PREFIX = 8 };

enum { FL_SINGLE = 0, FL_DIFFERENTIAL = 1 };

/* epilogue bits, applied in this order after normalisation by l_i (and after the differential
 * subtraction): RMSNorm over the Dv channels of a row (x * w / sqrt(mean(x^2) + rms_eps)),
 * then multiplication by sigmoid(gate).                                                      */
enum { FL_EPI_RMSNORM = 1, FL_EPI_GATE_SIGMOID = 2 };

typedef struct {
  uint32_t struct_size;    /* sizeof(fl_variant_desc) */
  float    scale;          /* multiplies <q,k>; 1/sqrt(D) for Eq. 3                           */
  uint32_t score_mod;      /* FL_MOD_*                                                        */
  float    softcap;        /* cap of cap*tanh(s/cap); > 0 when FL_MOD_SOFTCAP                 */
  uint32_t mask;           /* bit-or of FL_MASK_*                                             */
  int32_t  window;         /* >= 0 when FL_MASK_WINDOW                                        */
  int32_t  prefix_len;     /* >= 0 when FL_MASK_PREFIX                                        */
  uint32_t n_bias;         /* 0..2 additive bias tensors in aux->bias                         */
  uint32_t combine;        /* FL_SINGLE | FL_DIFFERENTIAL                                     */
  uint32_t epilogue;       /* bit-or of FL_EPI_*                                              */
  float    rms_eps;
  int32_t  q_offset;       /* >= 0: query row i sits at sequence position i + q_offset (key j at
                              position j): the positional masks and ALiBi use positions, so e.g.
                              q_offset = Sk - Sq aligns a causal mask bottom-right (a chunk of new
                              queries against a longer key/value cache, Sec. 4.1 serving).  Document
                              ids stay per row.  Forward and backward pass (not the decode step).   */
} fl_variant_desc;

typedef struct {
  uint32_t       struct_size;   /* sizeof(fl_aux) */
  uint32_t       reserved;
  const float*   alibi_slopes;  /* [H] device, FL_MOD_ALIBI                                    */
  const int32_t* q_doc_ids;     /* [B, Sq] device, contiguous, FL_MASK_DOC                     */
  const int32_t* kv_doc_ids;    /* [B, Sk] device, contiguous (may alias q_doc_ids)            */
  fl_tensor      bias[2];       /* logical [B, G, H, Sq, Sk]; stride 0 (or size 1) broadcasts;
                                   innermost stride 1 or 0; bf16 for bf16 inputs, bf16 or f32
                                   for f32 inputs; rows that start 8-byte aligned load faster  */
  fl_tensor      gate;          /* logical shape of out, pre-sigmoid; dtype of q               */
  fl_tensor      q2, k2;        /* second softmax stream (FL_DIFFERENTIAL); shapes of q, k     */
  const float*   lambda;        /* [H] device, FL_DIFFERENTIAL                                 */
  const float*   rms_weight;    /* [Dv] device, or NULL for all-ones                           */
  void*          workspace;     /* device scratch for the tile skipper (FL_MASK_DOC only)      */
  size_t         workspace_bytes;
} fl_aux;

/* The fused forward pass for the variant named by `desc`: the single kernel of Sec. 3 in which a
 * workgroup forms one tile of scaled scores at a time, folds it into a running row maximum and
 * row sum (rescaling what it has accumulated so far) and multiplies it by the matching V tile.
 *
 *   q    [B, G, H,   Sq, D ]  bf16 or f32 (all of q, k, v, q2, k2, gate share one dtype)
 *   k    [B, G, Hkv, Sk, D ]  Hkv divides H; query head h reads kv head h / (H / Hkv)
 *   v    [B, G, Hkv, Sk, Dv]
 *   out  [B, G, H,   Sq, Dv]  dtype of q, or f32
 *   lse  [B, G, H, Sq, 1] f32, or NULL / ptr == NULL to skip it.  For FL_DIFFERENTIAL the two
 *        streams' values go to axis G: size[1] must be 2*G, stream s of row-axis g at 2*g + s
 *        (with G = 1: lse[:, 0] is stream 1, lse[:, 1] is stream 2).
 *   aux  may be NULL when the descriptor needs nothing from it.
 *   stream  a hipStream_t (NULL = the default stream).
 *
 * A row whose keys are all masked gets out = 0 and lse = -inf.
 * Supported head dims: D, Dv in {32, 64, 128} for bf16 (the pairs listed by
 * fl_variant_supported), any multiple of 4 up to 128 for f32.  Sq, Sk >= 1 are arbitrary;
 * empty problems (any of B, G, H, Sq equal to 0) return FL_OK without a launch; Sk == 0 is
 * treated as every row fully masked.  (Grouped heads with fewer than 128 query rows against 1024 keys or more, the chunk
 * shape of q_offset: the query heads of a kv head share a workgroup; that kernel shape is compiled on the first such call.)
 * A call that compiles a kernel (a descriptor combination or shape outside the compiled table, first use in the process)
 * takes about a second on the host and loads a code object: make it once outside any stream capture.
 * Returns FL_OK or an error code; on error nothing was launched.                            */
fl_status fl_attn_fwd(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v,
                      const fl_variant_desc* desc, const fl_aux* aux,
                      fl_tensor* out, fl_tensor* lse, void* stream);

/* Bytes of aux->workspace that fl_attn_fwd needs for these shapes and this descriptor
 * (0 unless FL_MASK_DOC: the skipper's per-tile [min, max] document-id summaries; Sec. 4.3 notes
 * that the paper's own kernels do not skip masked blocks -- this goes beyond it).           */
size_t fl_attn_fwd_workspace_size(const fl_tensor* q, const fl_tensor* k,
                                  const fl_variant_desc* desc);

/* fl_attn_fwd for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, same kernels, same results, but the
 * tile skipper's document-id summaries (the only scratch of the forward pass, FL_MASK_DOC) go to a
 * buffer built into the library, 1 MiB per GPU, instead of aux->workspace; aux->workspace and
 * aux->workspace_bytes are ignored.  The call allocates and frees nothing.
 *
 *   limit   B * (ceil(Sq / 32) + ceil(Sk / 32)) * 8 bytes <= 1 MiB (e.g. B * (Sq + Sk) <= 4 Mi tokens);
 *           beyond it FL_ERR_WORKSPACE and nothing is launched.
 *   sharing every call on a GPU uses that GPU's one buffer: two such calls whose kernels may overlap
 *           in time (different streams, different host threads) race on it; calls on one stream are safe.
 *           The buffer is rewritten by every call, nothing in it has to be cleared in between.
 * Variants without FL_MASK_DOC need no scratch and behave exactly like fl_attn_fwd.          */
fl_status fl_attn_fwd_noalloc(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v,
                              const fl_variant_desc* desc, const fl_aux* aux,
                              fl_tensor* out, fl_tensor* lse, void* stream);

/* Gradient of fl_attn_fwd with respect to q, k and v, for the variants without bias, second
 * stream and epilogue (score_mod and every mask are covered).  The paper's conclusion names
 * training support as the extension it leaves open; this is the derivative of Eq. 3 with the
 * score_mod of Eq. 4 and the masks of the attention listing, evaluated like the forward pass
 * without materialising anything of size [Sq, Sk]: per score tile P = exp(s - lse) is recomputed
 * from the saved lse, dP = dout V^T, dS = P * (dP - rowsum(dout * out)) (times 1 - tanh^2 under a
 * soft-cap), and dv = P^T dout, dk = scale * dS^T q, dq = scale * dS k.
 *
 *   q, k, v      as given to fl_attn_fwd (bf16; D == Dv in {64, 128}; any score_mod and mask: a combination
 *                without a compiled backward kernel is instantiated on first use, as in the forward pass)
 *   out, lse     what fl_attn_fwd wrote for them: out [B, G, H, Sq, Dv] bf16, lse [B, G, H, Sq, 1] f32
 *   dout         [B, G, H, Sq, Dv] bf16, the gradient arriving at out
 *   dq           [B, G, H,   Sq, D ] bf16 or f32, written
 *   dk, dv       [B, G, Hkv, Sk, D ] bf16 or f32 (one dtype for both), written; with grouped
 *                query heads they hold the sum over the query heads of the group
 *   aux          required: aux->workspace of fl_attn_bwd_workspace_size bytes, 16-byte aligned
 *                (row statistics and tile-skipper summaries; contents undefined afterwards),
 *                plus alibi_slopes / doc ids as for the forward pass
 *
 * Rows without a visible key get dq = 0; keys that no row sees get dk = dv = 0.  Results are
 * bitwise reproducible (no atomics).  Same stream, ownership and error rules as fl_attn_fwd:
 * on an error code nothing was launched.                                                    */
fl_status fl_attn_bwd(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_tensor* out,
                      const fl_tensor* dout, const fl_tensor* lse, const fl_variant_desc* desc,
                      const fl_aux* aux, fl_tensor* dq, fl_tensor* dk, fl_tensor* dv, void* stream);

/* Bytes of aux->workspace that fl_attn_bwd needs for these shapes and this descriptor (variants without
 * bias, second stream and epilogue; for the others ask fl_attn_bwd_ex_workspace_size). */
size_t fl_attn_bwd_workspace_size(const fl_tensor* q, const fl_tensor* k, const fl_variant_desc* desc);

/* Gradient outputs beyond dq, dk, dv, for the variants whose forward pass reads more than q, k, v. */
typedef struct {
  uint32_t  struct_size;   /* sizeof(fl_bwd_extra) */
  uint32_t  reserved;
  fl_tensor dq2, dk2;      /* FL_DIFFERENTIAL: gradients of aux->q2 / aux->k2; shapes and dtypes as dq / dk; required */
  fl_tensor dbias[2];      /* gradient of aux->bias[n]: f32 with the sizes of aux->bias[n] (an axis of size 1 that
                              broadcasts holds the sum over that axis); ptr NULL: not computed.  The workspace then
                              holds dS of every score in bf16 ([B, G, H, Sq, Sk], 2 bytes each) until it is summed  */
  fl_tensor dgate;         /* FL_EPI_GATE_SIGMOID: gradient of aux->gate, shape of out, bf16 or f32; ptr NULL: not computed */
  float*    dlambda;       /* FL_DIFFERENTIAL: [H] f32 device; NULL: not computed                              */
  float*    drms_weight;   /* FL_EPI_RMSNORM: gradient of aux->rms_weight (of the implied all-ones weight when that is
                              NULL), [Dv] f32 device; NULL: not computed                                       */
} fl_bwd_extra;

/* fl_attn_bwd for every variant of the forward pass: additive biases (with their gradients), the sigmoid
 * gate, RMSNorm and the differential second stream, and the head dims the plain backward kernels do not
 * take (D = 32, D != Dv).  The derivative is that of the forward definition (differential listing; Evoformer
 * description in Sec. 4.1):
 *     dy = dout * sigmoid(g),  dg = dout * y * sigmoid(g) (1 - sigmoid(g))           gate
 *     dx = w dy / r - x (sum_c w_c dy_c x_c) / (Dv r^3),  r = sqrt(mean(x^2) + eps)  RMSNorm
 *     dw_c = sum over rows of dy_c x_c / r
 *     dO1 = dx,  dO2 = -lambda_h dx,  dlambda_h = -sum dx * O2                       x = O1 - lambda_h O2
 *     dbias = dS summed over the axes the bias broadcasts along
 * and then the softmax / contraction derivative of fl_attn_bwd per stream (dv sums both streams).
 * It is composed from the same kernels: the streams' outputs O1, O2 are recomputed with the forward kernel
 * where RMSNorm or the second stream need them, one elementwise kernel turns dout into the per-stream dO,
 * delta and the epilogue gradients, tensors whose head dim the backward kernels do not take are zero-padded
 * into the workspace (D = 32 -> 64, D = 64 with Dv = 128 -> 128), and the backward kernels run once per stream.
 *
 *   out, lse   what fl_attn_fwd wrote (lse [B, 2G, H, Sq, 1] for FL_DIFFERENTIAL)
 *   aux        as for fl_attn_fwd, with aux->workspace of fl_attn_bwd_ex_workspace_size bytes (16-byte aligned)
 *   extra      may be NULL when the variant has nothing beyond dq, dk, dv to write
 * Covered: every descriptor fl_attn_fwd takes for bf16 inputs (any score_mod with any mask, zero to two
 * biases, both epilogues, the second stream; D, Dv in {32, 64, 128}).  Variants outside the compiled table
 * of backward kernels are instantiated from the kernel templates on first use (hipRTC, a few seconds, once
 * per process and variant).
 * Same stream, ownership and error rules as fl_attn_fwd.                                  */
fl_status fl_attn_bwd_ex(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_tensor* out,
                         const fl_tensor* dout, const fl_tensor* lse, const fl_variant_desc* desc,
                         const fl_aux* aux, fl_tensor* dq, fl_tensor* dk, fl_tensor* dv,
                         const fl_bwd_extra* extra, void* stream);

/* Bytes of aux->workspace that fl_attn_bwd_ex needs. */
size_t fl_attn_bwd_ex_workspace_size(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v,
                                     const fl_variant_desc* desc);

/* 1 if fl_attn_bwd_ex (for the variants without bias, second stream and epilogue at D == Dv in {64, 128}:
 * also fl_attn_bwd) covers (descriptor, dtype, D, Dv), else 0. */
int fl_bwd_supported(const fl_variant_desc* desc, int dtype, int D, int Dv);

/* Where the cached keys and values of each sequence live (decode step). */
typedef struct {
  uint32_t       struct_size;   /* sizeof(fl_paged_kv) */
  uint32_t       reserved;
  const int32_t* block_table;   /* [B, table_stride] device: page holding tokens p*page_size .. of sequence b;
                                   NULL: no paging, sequence b is page b of the cache; an entry outside
                                   [0, pages) is cut to that range (wrong data, never a wild address)       */
  int32_t        table_stride;  /* elements between the rows of block_table                                  */
  int32_t        page_size;     /* tokens per page (size[3] of the cache tensors); with a block table a
                                   power of two >= 8                                                         */
  const int32_t* seq_lens;      /* [B] device: cached tokens of each sequence, 0 <= len <= pages * page_size */
  int32_t        max_seq_len;   /* host-side upper bound of seq_lens: sizes the launch and the workspace;
                                   a device length outside [0, max_seq_len] is cut to that range           */
  int32_t        reserved2;
} fl_paged_kv;

/* One decode step: for every sequence b, attention of its newest query rows over its len_b cached keys and
 * values -- the per-token call of the serving experiment in Sec. 4.1.  T = 1 is the token being generated (the
 * row at position len_b - 1); T > 1 are the T newest tokens (a speculative step's verification): row i sits at
 * position len_b - T + i and sees keys 0 .. that position, rows at negative positions (len_b < T) get out = 0
 * and lse = -inf.  Same arithmetic as fl_attn_fwd for those rows (Eq. 3, score_mod of Eq. 4, online softmax of
 * Sec. 3.4); the causal mask is implied, FL_MASK_WINDOW keeps each row's last window + 1 keys; other masks,
 * biases, the second stream and epilogues are FL_ERR_UNSUPPORTED.
 *
 *   q        [B, 1, H, T, D]  bf16, D in {64, 128}
 *   k_cache  [pages, 1, Hkv, page_size, D]  bf16, any strides with unit inner stride and 16-byte
 *   v_cache  [pages, 1, Hkv, page_size, D]  aligned rows (e.g. a view of [pages, page_size, Hkv, D]);
 *                                           Hkv divides H, T * H / Hkv <= 64 (else FL_ERR_SHAPE)
 *   out      [B, 1, H, T, D]  bf16 or f32;  lse [B, 1, H, T, 1] f32 or NULL
 *   aux      alibi_slopes for FL_MOD_ALIBI, and aux->workspace of fl_attn_decode_workspace_size bytes
 *            (per-split partial results; 16-byte aligned; contents undefined afterwards)
 *
 * A sequence with len = 0 gets out = 0 and lse = -inf.  The key range of a sequence is cut into
 * splits so that the launch fills the chip; the split count depends on B, Hkv and max_seq_len only,
 * and results are bitwise reproducible.  Stream, ownership and error rules as for fl_attn_fwd.   */
fl_status fl_attn_decode(const fl_tensor* q, const fl_tensor* k_cache, const fl_tensor* v_cache,
                         const fl_paged_kv* kv, const fl_variant_desc* desc, const fl_aux* aux,
                         fl_tensor* out, fl_tensor* lse, void* stream);

/* Bytes of aux->workspace that fl_attn_decode needs. */
size_t fl_attn_decode_workspace_size(const fl_tensor* q, const fl_tensor* k_cache, const fl_paged_kv* kv);

/* A chunk of Sq query rows per sequence against that sequence's paged cache: the prompt phase of the
 * serving experiment in Sec. 4.1 (time to first token) when a prompt is processed in chunks or continues a
 * cached prefix.  The chunk's own keys and values are already in the cache: query row i of sequence b is the
 * token at position len_b - Sq + i and attends to keys 0 .. that position (the causal mask is implied;
 * FL_MASK_WINDOW keeps the last window + 1 of them), with the arithmetic of fl_attn_fwd (Eq. 3, score_mod of
 * Eq. 4, online softmax of Sec. 3.4).  Rows at negative positions (len_b < Sq) get out = 0 and lse = -inf.
 * Sq = 1 computes what fl_attn_decode computes.
 *
 *   q        [B, 1, H, Sq, D]  bf16, D in {32, 64, 128}
 *   k_cache, v_cache, kv       as for fl_attn_decode (Hkv divides H; no limit on H / Hkv)
 *   out      [B, 1, H, Sq, D]  bf16 or f32;  lse [B, 1, H, Sq, 1] f32 or NULL
 *   desc     scale, score_mod, FL_MASK_CAUSAL and / or FL_MASK_WINDOW (or no mask bit: causal all the same);
 *            other masks, biases, the second stream, epilogues and q_offset are FL_ERR_UNSUPPORTED
 *   aux      alibi_slopes for FL_MOD_ALIBI, and aux->workspace of fl_attn_prefill_paged_workspace_size bytes
 *            (16-byte aligned; contents undefined afterwards); may be NULL when neither is needed
 *
 * How: chunks of so few rows that Sq * H / Hkv <= 32 (D 64 or 128; <= 64 when the forward kernel would not fill the chip)
 * are an fl_attn_decode call on the same arguments (the cache is then read once per kv head; the workspace is that call's).  Otherwise the forward kernel runs with each
 * sequence's length read on the device: it stops at that length and places the
 * query rows at its last Sq positions (for chunks much shorter than its 128- or 256-row tiles a workgroup takes the rows
 * of several query heads of one kv head), so a short sequence costs its own length and nothing is synchronised with the
 * host.  For chunks of up to 1024 rows its key / value tile loads go to the pages themselves (page numbers from the block
 * table, fetched a step ahead; needs page_size >= 512 / D with a block table): no copy and no workspace.  For longer
 * chunks one pass first copies the cached rows of every sequence into dense tensors in the workspace (2 * 2 * len * Hkv
 * * D * 2 bytes read and written per sequence, small beside the Sq * len scores of such a chunk) and the tuned dense
 * kernel runs on those.  fl_attn_prefill_paged_workspace_size says which: 0 for reading in place.
 * Stream, ownership and error rules as for fl_attn_fwd.                                                  */
fl_status fl_attn_prefill_paged(const fl_tensor* q, const fl_tensor* k_cache, const fl_tensor* v_cache,
                                const fl_paged_kv* kv, const fl_variant_desc* desc, const fl_aux* aux,
                                fl_tensor* out, fl_tensor* lse, void* stream);

/* Bytes of aux->workspace that fl_attn_prefill_paged needs: fl_attn_decode_workspace_size for chunks of a few rows,
 * 0 when the forward kernel reads the pages in place, else the dense copies, 2 * B * Hkv * max_seq_len * D * 2 bytes
 * (each rounded up to 256). */
size_t fl_attn_prefill_paged_workspace_size(const fl_tensor* q, const fl_tensor* k_cache, const fl_paged_kv* kv);

/* A variant compiled at run time from user expressions (opaque; owned by the caller until released). */
typedef struct fl_custom_variant fl_custom_variant;

/* Compiles (hipRTC, a few seconds) the forward kernel for a variant that the descriptor cannot
 * name -- the library's stand-in for the paper's compiler accepting an arbitrary attention program:
 *   score_mod_expr  C expression for the new score, of: float s (the scaled score, Eq. 4),
 *                   int b, g, h (batch, row axis, query head), int i, j (query and key index);
 *                   e.g. "s - 0.25f * fabsf((float)(i - j))".  NULL: s.
 *   mask_expr       C expression, nonzero where the score is replaced by -inf (the mask_mod of
 *                   Sec. 2.2, inverted), of int b, g, h, i, j; e.g. "j > i || (i - j) % 4 != 0".
 *                   NULL: nothing masked.  It is evaluated on every score: no tile is skipped.
 *   base_mask       FL_MASK_CAUSAL / FL_MASK_WINDOW / FL_MASK_PREFIX bits OR-ed into the mask: these the
 *                   kernel knows in closed form, so tiles they hide are skipped and tiles they leave
 *                   fully visible skip the mask arithmetic (when there is no mask_expr).
 *   D               head dim (= Dv), 64 or 128; bf16 inputs.  (At 128 the kernel takes 256 query rows per
 *                   workgroup on eight waves, at 64 it takes 128 rows on four.)
 * An expression is one C expression (no ; { } # quotes or backslashes).  FL_ERR_DESC with the
 * compiler's first error in fl_last_error_detail() if it does not compile.  Needs no GPU.       */
fl_status fl_compile_variant(const char* score_mod_expr, const char* mask_expr, uint32_t base_mask, int D,
                             fl_custom_variant** handle);

/* The forward pass of a compiled variant: q, k, v, out, lse, stream as for fl_attn_fwd (grouped
 * heads included); window / prefix_len belong to the base mask (ignored without it).  The code
 * object is loaded on the current device at the first call there.                              */
fl_status fl_attn_fwd_custom(fl_custom_variant* variant, const fl_tensor* q, const fl_tensor* k, const fl_tensor* v,
                             float scale, int32_t window, int32_t prefix_len, fl_tensor* out, fl_tensor* lse,
                             void* stream);

/* fl_compile_variant for expressions that read caller-supplied device arrays, as the score_mod / mask_mod
 * closures of Sec. 2.2 capture tensors (the per-token document ids of the document mask of Sec. 4.1, a
 * learned relative-position bias table, per-head slopes): inside both expressions
 *   aux0 .. aux3   are pointers to the arrays given at call time, typed by aux_dtypes[n]:
 *                  FL_I32 -> const int*, FL_F32 -> const float*, FL_BF16 -> elements that read as float;
 *                  0 -> that name does not exist.  Index arithmetic is the expression's own, e.g.
 *                  mask_expr "aux0[b * Sq + i] != aux1[b * Sk + j]", score_mod_expr "s + aux2[h * 64 + min(i - j, 63)]".
 *   B, G, H, Sq, Sk  are the sizes of the call.
 * aux_dtypes may be NULL (no arrays: the same as fl_compile_variant).  The library cannot check what an
 * expression indexes: an out-of-range index is the caller's error, as in any kernel the caller writes.  */
fl_status fl_compile_variant_aux(const char* score_mod_expr, const char* mask_expr, uint32_t base_mask, int D,
                                 const int32_t* aux_dtypes, fl_custom_variant** handle);

/* fl_attn_fwd_custom with the arrays the variant's expressions read: aux_ptrs[n] is a DEVICE pointer for every
 * n whose dtype was given at compile time (FL_ERR_AUX_MISSING otherwise); the other entries are ignored.  */
fl_status fl_attn_fwd_custom_aux(fl_custom_variant* variant, const fl_tensor* q, const fl_tensor* k, const fl_tensor* v,
                                 float scale, int32_t window, int32_t prefix_len, const void* const* aux_ptrs,
                                 fl_tensor* out, fl_tensor* lse, void* stream);

/* fl_attn_fwd_custom_aux with tile skipping for the mask expression (the block sparsity that the mask_mod of
 * Sec. 2.2 allows; Sec. 4.3 notes that the paper's own kernels evaluate every block).  A pre-pass, compiled with the
 * variant, evaluates the whole mask (base_mask and mask_expr) once per score and writes one class byte per
 * (32 query rows, 64 keys) into the workspace: nothing visible / some / all, and (while Sq * Sk / 8 bytes per
 * problem stay under 1 GiB in all) one bit per score; the attention kernel then passes over tiles with nothing
 * visible to its workgroup, does not mask tiles that are all visible, and on the others applies the stored bits
 * instead of evaluating the expression.  Same results as fl_attn_fwd_custom_aux.  The pre-pass runs in every call (the arrays an expression reads may have
 * changed); it is per batch element unless the expression reads g or h, then per (b, g, h).
 *   workspace   DEVICE, fl_custom_skip_workspace_size bytes, 16-byte aligned; contents undefined afterwards
 * A variant without a mask expression needs no workspace and behaves like fl_attn_fwd_custom_aux.  */
fl_status fl_attn_fwd_custom_skip(fl_custom_variant* variant, const fl_tensor* q, const fl_tensor* k, const fl_tensor* v,
                                  float scale, int32_t window, int32_t prefix_len, const void* const* aux_ptrs,
                                  void* workspace, size_t workspace_bytes, fl_tensor* out, fl_tensor* lse, void* stream);

/* Bytes of workspace that fl_attn_fwd_custom_skip needs for these shapes (0 without a mask expression). */
size_t fl_custom_skip_workspace_size(fl_custom_variant* variant, const fl_tensor* q, const fl_tensor* k);

/* fl_compile_variant_aux for callers who also want the backward pass of the variant (the paper leaves training as future
 * work; this extends its "arbitrary attention program" to the gradient):
 *   score_mod_grad_expr  C expression for the derivative of score_mod_expr with respect to s, of the same names
 *                        (s, b, g, h, i, j, aux0 .. aux3, B, G, H, Sq, Sk); NULL: 1, which is right for every score_mod of
 *                        the form s + f(b, g, h, i, j) (relative biases, ALiBi-like terms).  E.g. for
 *                        "8.0f * tanhf(s / 8.0f)": "1.0f - tanhf(s / 8.0f) * tanhf(s / 8.0f)".
 * With a derivative expression the backward kernels are compiled here too (a few seconds more), so that an error in it
 * is reported by this call; without one they are compiled by the first fl_attn_bwd_custom call.            */
fl_status fl_compile_variant_grad(const char* score_mod_expr, const char* score_mod_grad_expr, const char* mask_expr,
                                  uint32_t base_mask, int D, const int32_t* aux_dtypes, fl_custom_variant** handle);

/* Gradients of a compiled variant with respect to q, k, v: fl_attn_bwd with the variant's score_mod (and its derivative
 * expression) and mask in place of the descriptor's.  out, lse: what fl_attn_fwd_custom[_aux | _skip] wrote; dout, dq, dk,
 * dv, the stream and the error rules as for fl_attn_bwd; scale, window, prefix_len, aux_ptrs as in the forward call.
 * The mask expression is evaluated on every score of every tile inside the base mask's range (no tile-class map here).
 *   workspace   DEVICE, fl_attn_bwd_custom_workspace_size bytes, 16-byte aligned; contents undefined afterwards   */
fl_status fl_attn_bwd_custom(fl_custom_variant* variant, const fl_tensor* q, const fl_tensor* k, const fl_tensor* v,
                             const fl_tensor* out, const fl_tensor* dout, const fl_tensor* lse, float scale,
                             int32_t window, int32_t prefix_len, const void* const* aux_ptrs, void* workspace,
                             size_t workspace_bytes, fl_tensor* dq, fl_tensor* dk, fl_tensor* dv, void* stream);

/* Bytes of workspace that fl_attn_bwd_custom needs for these shapes. */
size_t fl_attn_bwd_custom_workspace_size(fl_custom_variant* variant, const fl_tensor* q, const fl_tensor* k);

/* Unloads and frees a compiled variant (no launch of it may be in flight). */
void fl_release_variant(fl_custom_variant* variant);

/* 1 if a kernel specialisation exists for (descriptor, dtype, D, Dv), else 0. */
int fl_variant_supported(const fl_variant_desc* desc, int dtype, int D, int Dv);

/* Static text for a status code. */
const char* fl_strerror(fl_status status);

/* Thread-local detail of the last failure in this thread (which check failed, or the HIP error
 * string); valid until the next library call of the thread.                                 */
const char* fl_last_error_detail(void);

/* Tuning knobs for benchmarking sweeps: choose a non-default kernel shape among the compiled
 * ones.  `key` is one of "bm" (query rows per workgroup), "bn" (keys per tile), "nw" (waves per
 * workgroup), "rb" (32-row blocks per wave), "wpe" (waves per SIMD the kernel is built for), "ring" (slots of
 * the K / V rings in LDS: 2 = a workgroup barrier per key tile, 4 = one per two tiles),
 * "order" (1 = plain, 2 = XCD-aware workgroup order), "pair" (1 = one q-tile per workgroup,
 * 2 = a long and a short q-tile per workgroup), "decode_splits" (key-range splits per sequence and
 * kv head of fl_attn_decode), "bwd_wg_target" (workgroups up to which fl_attn_bwd cuts a group of
 * query heads into subsets; both change the workspace size the matching *_workspace_size reports),
 * "prefill_gather" (fl_attn_prefill_paged: 1 = always copy the pages first, 2 = always read them in place with the
 * forward kernel; either also keeps chunks of a few rows away from the decode kernels), "prefill_pack" (1 = never
 * pack the query heads of a kv head into one workgroup of the in-place kernel).
 * Value 0 restores the built-in choice.  Returns FL_OK or FL_ERR_UNSUPPORTED.  The requests are kept
 * per host thread: they change the later calls of the calling thread only, so this call is as
 * thread-safe as the others and no state is shared between threads.                          */
fl_status fl_set_tuning(const char* key, int value);

/* ABI version: major << 16 | minor. */
uint32_t fl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FL_ATTN_H */
