/*
 * massv_verify.h -- C ABI of the target-model verify step of speculative decoding
 * for AMD MI355X (gfx950).
 *
 * One iteration of speculative decoding (MASSV paper, Section 2.1): a drafter
 * proposes gamma tokens; the target model scores those gamma tokens plus one
 * further position in ONE parallel forward pass; the drafts are then examined
 * in order, each accepted with probability min(1, p/q), the first rejection is
 * replaced by a draw from norm(max(p - q, 0)) and ends the iteration; at
 * temperature 0 a draft is accepted iff it equals argmax p and a rejected one
 * is replaced by argmax p.  This library is the target's half of that
 * iteration: the parallel forward (decoder layers, vocabulary projection) and
 * the accept / resample rule.
 *
 * Conventions common to every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The
 *     library never allocates, frees or synchronises; a call only enqueues
 *     kernels on `stream` (a hipStream_t passed as void*, NULL = the null
 *     stream).  Scratch space is the caller's `workspace`, whose minimum size
 *     the matching *_workspace() function returns; it need not be zeroed and
 *     holds nothing between calls.  Descriptor structs are HOST pointers and
 *     are read before the call returns.
 *   - Return value: MASSV_OK or a negative massv_status.  Arguments are
 *     validated on the host before anything is enqueued; on MASSV_EINVAL,
 *     MASSV_EUNSUPPORTED and MASSV_EWORKSPACE nothing has been launched.
 *     Values held in device memory (kv_len, tokens) cannot be checked without
 *     a synchronisation; kernels clamp them so that no access leaves the
 *     buffers described by the descriptor, but results are then unspecified.
 *   - Calls are stateless; the same inputs give bit-identical outputs (no
 *     floating-point atomics, reductions in a fixed order).
 *   - Notation: B batch, gamma speculation length, Q = gamma+1 query positions,
 *     M = B*Q rows, H hidden, n_q / n_kv query / KV heads, G = n_q/n_kv,
 *     d head_dim, F MLP width, V vocabulary, L_b = kv_len[b] = cached length of
 *     sequence b BEFORE the step, L_max = rows allocated per sequence.
 *
 * KV cache layout (dtype = f32 or bf16 elements)
 *   k_cache, f32   [B][n_kv][L_max][d]     row j of (b, g) at ((b*n_kv+g)*L_max + j)*d
 *   k_cache, bf16  [B][n_kv][L_max/32][2][d/8][16][8]: the 32 rows of a block form two halves of 16; row
 *                  jj of the block is slot 4*(jj/8) + jj%4 of half (jj/4)%2, and a half is stored by
 *                  8-feature chunks, the 16 slots of a chunk back to back.  Element (j, c) of (b, g) at
 *                    ((b*n_kv+g)*L_max + 32*(j/32))*d + (((j/4)%2*(d/8) + c/8)*16 + 4*((j%32)/8) + j%4)*8 + c%8
 *                  This is the order in which the score product's matrix instruction takes its key
 *                  operand, so a wavefront reads 1 KB of whole cache lines per load; with row-major keys
 *                  every load touched 16 half lines.  massv_k_cache_pack() converts from row-major.
 *   v_cache [B][n_kv][L_max/32][d][32]     element (j, c) of (b, g) at
 *                                          (((b*n_kv+g)*(L_max/32) + j/32)*d + c)*32 + j%32
 *   L_max must be a multiple of 32.  Values are stored key-minor in blocks of
 *   32 keys so that the probability-times-value product reads them in matrix
 *   operand order with 16-byte loads.  massv_v_cache_pack() converts a
 *   row-major [B][n_kv][L_max][d] tensor into this layout.
 *   The leading rows of a sequence's cache are its image-token positions
 *   followed by text positions (Section 2.2); the kernels treat both alike.
 *
 * Weight layout
 *   Every projection matrix W[N][K] (wq, wk, wv, wo, wg, wu, wd, w_lm) is passed in the library's
 *   STREAMING layout, produced once per matrix by massv_weight_pack() from the usual row-major
 *   [out][in] tensor (weights are static during decoding, so this is a load-time step):
 *     f32   row-major, unchanged;
 *     bf16  [N/16][K/32][64][8]: for each tile of 16 output features and each step of 32 inputs, the
 *           64 lanes' matrix-instruction operands back to back -- element (n, k) at
 *           (((n/16)*(K/32) + k/32)*64 + (n%16) + 16*((k%32)/8))*8 + k%8 -- so that a wavefront
 *           streams a tile as one contiguous run of whole cache lines.  Needs N % 16 == 0, K % 32 == 0.
 *   Norm gains and biases are plain vectors.
 */
#ifndef MASSV_VERIFY_H
#define MASSV_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MASSV_OK = 0,
    MASSV_EINVAL = -1,        /* NULL pointer, non-positive size, n_q % n_kv != 0, T < 0 or NaN ... */
    MASSV_EUNSUPPORTED = -2,  /* valid but outside what the kernels are built for */
    MASSV_EWORKSPACE = -3,    /* workspace NULL or smaller than *_workspace() says */
    MASSV_ELAUNCH = -4        /* the HIP runtime refused a launch */
} massv_status;

typedef enum { MASSV_F32 = 0, MASSV_BF16 = 1 } massv_dtype;
typedef enum { MASSV_ACT_SILU = 0, MASSV_ACT_GELU_TANH = 1 } massv_act;

#define MASSV_V_BLOCK 32          /* keys per block of the value cache */
#define MASSV_MAX_ROWS 64         /* largest M = B*Q (and G*Q) the bf16 kernels take */

/* Text for a status code; never NULL.  Host pointer to static storage. */
const char* massv_status_string(int status);
/* ABI version, bumped when a signature or layout changes. */
int massv_abi_version(void);

/* ------------------------------------------------------------------------- */
/* verify_attention: grouped-query causal attention of the Q new positions.   */
/* Section 2.1: position i of the parallel forward conditions on all earlier  */
/* positions, so query i (0-based) attends to cache rows [0, L_b + i], the    */
/* new positions' own keys included (they must already be in the cache at     */
/* rows L_b .. L_b+Q-1).  Query head h reads KV head h / G.                   */
/*   out[b,i,h,:] = sum_j softmax_j(scale * q[b,i,h,:].k[b,h/G,j,:]) v[b,h/G,j,:] */
/* window = W > 0 restricts query i to the last W of those rows,               */
/* [max(0, L_b+i-W+1), L_b+i]: the sliding-window layers of the Gemma 3        */
/* targets named in Section 5 ("Models"); rows before the window of the first  */
/* query are not read at all.                                                  */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t batch;            /* B >= 1 */
    int32_t n_query;          /* Q = gamma+1 >= 1 */
    int32_t n_q_heads;
    int32_t n_kv_heads;       /* divides n_q_heads */
    int32_t head_dim;         /* f32: multiple of 2, <= 256; bf16: 64, 128 or 256 */
    int32_t l_max;            /* rows allocated per (b, kv head); multiple of 32 */
    float   scale;            /* 0 => 1/sqrt(head_dim) */
    int32_t dtype;            /* massv_dtype of q, caches and out */
    int32_t window;           /* 0: every cached row; W > 0: the last W rows only */
} massv_attn_desc;

/* Bytes of workspace massv_verify_attention needs for this descriptor (0 if the
 * descriptor is invalid). */
size_t massv_verify_attention_workspace(const massv_attn_desc* desc);

/* q   [B][Q][n_q][d]  (dtype)   in
 * k_cache, v_cache    (dtype)   in, layouts above; rows [0, kv_len[b]+Q) valid
 * kv_len [B] int32              in, 0 <= kv_len[b], kv_len[b]+Q <= l_max (caller's duty)
 * out [B][Q][n_q][d]  (dtype)   out
 * bf16 path requires G*Q <= MASSV_MAX_ROWS, else MASSV_EUNSUPPORTED. */
int massv_verify_attention(const massv_attn_desc* desc, const void* q,
                           const void* k_cache, const void* v_cache,
                           const int32_t* kv_len, void* out,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- */
/* prefill_attention: the same attention for the prompt pass that fills the    */
/* cache.  Section 2.2: the m projected image features V_1..V_m enter the      */
/* sequence ahead of the text tokens and the language model conditions on all  */
/* of them; here they are rows of the cache like any other position.  Sequence */
/* b brings n_new[b] <= L_q new positions (their keys and values already at    */
/* cache rows kv_len[b] .. kv_len[b]+n_new[b]-1; kv_len[b] > 0 when a prompt   */
/* is fed in several pieces); the query at cache row r sees rows 0 .. r, with  */
/* desc->window = W > 0 rows max(0, r-W+1) .. r only.  n_bidir (may be NULL):  */
/* n_bidir[b] = m makes the first m cache rows of sequence b a block whose     */
/* members see the whole block (a query at row r < m sees rows 0 .. m-1), the  */
/* way the Gemma 3 family treats an image's positions; the paper itself does   */
/* not say, the default is causal.                                             */
/*   desc: n_query = L_q (rows allocated per sequence in q and out), the other */
/*         fields as for verify_attention; no limit on G*L_q.  No workspace.   */
/*   q, out [B][L_q][n_q][d] (dtype); rows i >= n_new[b] of out are not        */
/*   written.  Caches in the layouts above.  kv_len, n_new, n_bidir [B] int32  */
/*   device; kv_len[b] + n_new[b] <= l_max is the caller's duty (clamped).     */
/* ------------------------------------------------------------------------- */
int massv_prefill_attention(const massv_attn_desc* desc, const void* q,
                            const void* k_cache, const void* v_cache,
                            const int32_t* kv_len, const int32_t* n_new, const int32_t* n_bidir,
                            void* out, void* stream);

/* ------------------------------------------------------------------------- */
/* rope_append: the step of the prompt pass between the q/k/v projection and   */
/* prefill_attention (Section 2.2: image features, then text, enter the        */
/* sequence as positions).  The projected rows are split into heads, query and */
/* key heads optionally normalised (q_norm, k_norm [d], may be NULL; as in the */
/* layer), queries and keys rotated by their position ids in the half-split    */
/* pairing (j, j + d/2), and the keys and values of the first n_new[b] rows of */
/* sequence b written into the caches at rows kv_len[b] + i.                   */
/* Position ids: n_pos = 1, pos [B][L_q]: pair j turns by pos * theta^(-2j/d). */
/* n_pos = 3, pos [3][B][L_q] (temporal, height, width ids, the numbering the  */
/* Qwen2.5-VL targets of Section 5 give image positions; text positions carry  */
/* three equal ids) and sections = three HOST int32 pair counts summing to     */
/* d/2: pairs [0, s0) turn by the temporal id, the next s1 by the height id,   */
/* the last s2 by the width id, each at its own frequency theta^(-2j/d).       */
/*   desc: n_query = L_q rows per sequence in qkv, pos and q_out; heads,       */
/*         head_dim, l_max, dtype as for verify_attention; no limit on L_q.    */
/*   qkv   [B][L_q][(n_q + 2 n_kv) d] (dtype) in: query, key, value heads      */
/*   q_out [B][L_q][n_q][d] (dtype) out; rows i >= n_new[b] are not written    */
/*   k_cache, v_cache in/out, layouts above; rows outside                      */
/*         [kv_len[b], kv_len[b] + n_new[b]) are not touched                   */
/*   kv_len, n_new [B] int32 device; kv_len[b] + n_new[b] <= l_max is the      */
/*         caller's duty (clamped).  No workspace.                             */
/* MASSV_EINVAL: NULL pointers, n_pos not 1 or 3, sections missing, negative   */
/* or not summing to d/2, theta <= 0.                                          */
/* ------------------------------------------------------------------------- */
int massv_rope_append(const massv_attn_desc* desc, const void* qkv, const int32_t* pos, int32_t n_pos,
                      const int32_t* sections, float rope_theta, const void* q_norm, const void* k_norm,
                      float norm_eps, const int32_t* kv_len, const int32_t* n_new, void* q_out,
                      void* k_cache, void* v_cache, void* stream);

/* Row-major [B][n_kv][L_max][d] values -> blocked value-cache layout. src and
 * dst must not overlap. */
int massv_v_cache_pack(const void* src_row_major, void* dst_blocked,
                       int32_t batch, int32_t n_kv_heads, int32_t l_max, int32_t head_dim,
                       int32_t dtype, void* stream);

/* Row-major [B][n_kv][L_max][d] keys -> key-cache layout of this dtype (f32: a plain copy; bf16: the blocked
 * order above, needs L_max % 32 == 0 and d % 8 == 0).  src and dst must not overlap. */
int massv_k_cache_pack(const void* src_row_major, void* dst,
                       int32_t batch, int32_t n_kv_heads, int32_t l_max, int32_t head_dim,
                       int32_t dtype, void* stream);

/* Row-major W[N][K] -> streaming layout (see "Weight layout").  src and dst hold N*K elements and
 * must not overlap.  bf16: MASSV_EUNSUPPORTED unless N % 16 == 0 and K % 32 == 0. */
int massv_weight_pack(const void* src_row_major, void* dst, int32_t N, int32_t K, int32_t dtype, void* stream);

/* ------------------------------------------------------------------------- */
/* verify_layer: one pre-norm decoder layer of the parallel forward over the  */
/* M = B*Q new positions (the single forward pass of Section 2.1; the paper    */
/* does not spell the layer out -- this is the usual gated-MLP block):         */
/*   xn = rmsnorm(x, ln1);  q,k,v = xn Wq^T+bq, xn Wk^T+bk, xn Wv^T+bv         */
/*   q,k = rope(q,k; pos);  cache rows L_b+i <- k,v;  a = attention(q, cache)  */
/*   h = x + a Wo^T;  hn = rmsnorm(h, ln2)                                     */
/*   x <- h + (act(hn Wg^T) * (hn Wu^T)) Wd^T                                  */
/* rmsnorm(x,g) = x * g / sqrt(mean(x^2) + eps).  rope rotates the pairs       */
/* (j, j + d/2) of every head by angle pos * theta^(-2j/d).                    */
/* Optional steps of the Gemma 3 family (Section 5's 12B / 27B targets), each  */
/* switched on by a non-NULL gain vector in massv_layer_weights:               */
/*   q_norm, k_norm [d]:  every query / key head is replaced by its rmsnorm    */
/*                        over head_dim (after the bias, before rope);        */
/*   post_attn_norm [H]:  h = x + rmsnorm(a Wo^T, post_attn_norm);             */
/*   post_mlp_norm [H]:   x <- h + rmsnorm(mlp output, post_mlp_norm).         */
/* ------------------------------------------------------------------------- */
typedef struct {
    massv_attn_desc attn;     /* batch, n_query, heads, head_dim, l_max, scale, dtype */
    int32_t hidden;           /* H */
    int32_t mlp;              /* F */
    int32_t act;              /* massv_act */
    int32_t qkv_bias;         /* 0: bq,bk,bv ignored (may be NULL) */
    float   norm_eps;
    float   rope_theta;
} massv_layer_desc;

/* All weights are DEVICE pointers of the layer's dtype; matrices in the streaming layout of
 * massv_weight_pack(), shapes given as [out][in]. */
typedef struct {
    const void* ln1;          /* [H] */
    const void* wq;           /* [n_q*d][H] */
    const void* wk;           /* [n_kv*d][H] */
    const void* wv;           /* [n_kv*d][H] */
    const void* bq;           /* [n_q*d] or NULL */
    const void* bk;           /* [n_kv*d] or NULL */
    const void* bv;           /* [n_kv*d] or NULL */
    const void* wo;           /* [H][n_q*d] */
    const void* ln2;          /* [H] */
    const void* wg;           /* [F][H] */
    const void* wu;           /* [F][H] */
    const void* wd;           /* [H][F] */
    const void* q_norm;       /* [d] or NULL */
    const void* k_norm;       /* [d] or NULL */
    const void* post_attn_norm; /* [H] or NULL */
    const void* post_mlp_norm;  /* [H] or NULL */
} massv_layer_weights;

size_t massv_verify_layer_workspace(const massv_layer_desc* desc);

/* x   [B][Q][H] (dtype)  in/out: the residual stream, updated in place
 * pos [B][Q] int32       in: rotary position id of each new token (need not
 *                        equal its cache row: image prefixes may be numbered
 *                        differently from the rows they occupy)
 * k_cache, v_cache       in/out: rows kv_len[b]+i (i < Q) are written, then
 *                        rows [0, kv_len[b]+Q) are read
 * kv_len [B] int32       in
 * bf16 path requires M <= MASSV_MAX_ROWS, H, F, n_q*d multiples of 32 and
 * every projection's output size a multiple of 16. */
int massv_verify_layer(const massv_layer_desc* desc, const massv_layer_weights* weights,
                       void* x, const int32_t* pos, void* k_cache, void* v_cache,
                       const int32_t* kv_len,
                       void* workspace, size_t workspace_bytes, void* stream);

/* The same for n_layers consecutive layers that share one descriptor (a whole model's stack, or a
 * slice of it): weights[l], k_caches[l], v_caches[l] belong to layer l; `weights`, `k_caches`,
 * `v_caches` are HOST arrays (of structs / of device pointers) read before the call returns.  Equal to
 * n_layers calls of massv_verify_layer, except that the norm opening layer l+1 is computed by the kernel
 * that closes layer l from its un-rounded sum (one launch fewer per layer).  Workspace as for one layer.
 * windows, rope_thetas: HOST arrays [n_layers] that replace desc->attn.window / desc->rope_theta for
 * layer l (stacks that interleave sliding-window and global layers), or NULL to use the descriptor's
 * values for every layer. */
int massv_verify_layers(const massv_layer_desc* desc, const massv_layer_weights* weights, int32_t n_layers,
                        void* x, const int32_t* pos, void* const* k_caches, void* const* v_caches,
                        const int32_t* kv_len, const int32_t* windows, const float* rope_thetas,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- */
/* lm_head_logits: logits[m, v] = sum_k rmsnorm(x, final_norm)[m, k] * w_lm[v, k] */
/* (no norm when final_norm == NULL).  Row i of sequence b gives the scores   */
/* from which p_{i+1}( . | ...) of Section 2.1 is formed.                      */
/* ------------------------------------------------------------------------- */
size_t massv_lm_head_logits_workspace(int32_t M, int32_t H, int32_t V, int32_t dtype);

/* x [M][H] (dtype) in; final_norm [H] (dtype) or NULL; w_lm [V][H] (dtype, streaming layout) in;
 * logits [M][V] float32 out.  bf16 path: M <= MASSV_MAX_ROWS, H % 32 == 0, V % 16 == 0. */
int massv_lm_head_logits(const void* x, const void* final_norm, const void* w_lm,
                         float* logits, int32_t M, int32_t H, int32_t V,
                         float norm_eps, int32_t dtype,
                         void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- */
/* spec_accept: the sequential accept / reject / resample rule of Section 2.1  */
/* for every sequence of the batch.                                           */
/*   T > 0: p_i = softmax(target_logits[b,i]/T), q_i = softmax(draft_logits[b,i]/T); */
/*          draft x_i (i = 0..gamma-1, examined in order) is accepted iff      */
/*          p_i(x_i) >= q_i(x_i) or uniforms[b,i] * q_i(x_i) < p_i(x_i);        */
/*          at the first rejection (index n) the final token is the smallest k */
/*          with sum_{x<=k} r_x > uniforms[b,gamma] * sum_x r_x,                */
/*          r = max(p_n - q_n, 0) (r = p_n if that is identically zero);        */
/*          if all gamma are accepted (n = gamma) the same draw with r = p_gamma. */
/*   T = 0: x_i accepted iff x_i == argmax target_logits[b,i] (lowest index on */
/*          ties); final token = argmax target_logits[b,n].                    */
/* After the call the caller keeps kv_len[b] + n_accepted[b] + 1 cache rows.   */
/* gamma = 0 is the plain sampling step of the drafting loop (Section 2.1: the */
/* drafter draws x_i from q_i): there is nothing to verify, n_accepted = 0 and */
/* out_tokens[b,0] is drawn from softmax(target_logits[b,0]/T) with            */
/* uniforms[b,0] (argmax at T = 0); draft_logits and draft_tokens are unused.  */
/* ------------------------------------------------------------------------- */
size_t massv_spec_accept_workspace(int32_t B, int32_t gamma, int32_t V);

/* target_logits [B][gamma+1][V] float32 in
 * draft_logits  [B][gamma][V]   float32 in; may be NULL iff temperature == 0 or gamma == 0
 * draft_tokens  [B][gamma]      int32   in; values outside [0,V) are rejected; may be NULL iff gamma == 0
 * uniforms      [B][gamma+1]    float32 in, in [0,1); may be NULL iff temperature == 0
 * n_accepted    [B]             int32   out, 0..gamma
 * out_tokens    [B][gamma+1]    int32   out: the accepted drafts, the final
 *                                       token, then -1 padding
 * Logits must not contain NaN or +inf (-inf is a zero-probability token). */
int massv_spec_accept(const float* target_logits, const float* draft_logits,
                      const int32_t* draft_tokens, const float* uniforms,
                      float temperature, int32_t B, int32_t gamma, int32_t V,
                      int32_t* n_accepted, int32_t* out_tokens,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- */
/* spec_accept_static: massv_spec_accept for callers that cannot allocate or   */
/* carry a workspace -- code under HIP graph capture, tight serving loops,     */
/* harnesses that forbid hipMalloc.  Same arguments without the workspace,     */
/* same kernels, bit-identical results.  The partial results of the call       */
/* (per-chunk row statistics, the per-sequence selection records, per-chunk    */
/* residual masses) live in a fixed array of MASSV_SPEC_ACCEPT_STATIC_BYTES of */
/* device memory inside the library; every GPU the library is used on holds    */
/* its own copy until the process ends.  The call allocates and frees nothing. */
/*   - Sizes whose scratch need, massv_spec_accept_workspace(B, gamma, V),     */
/*     exceeds the array return MASSV_EUNSUPPORTED before anything is launched */
/*     (the long-context shape B=32, gamma=7, V=152064 needs 1.2 MB).          */
/*   - All calls on one GPU share that GPU's array: calls that overlap in time */
/*     on one GPU (two streams, two threads) race; serialise them.  The array  */
/*     keeps the last call's contents; nothing in it needs clearing, every     */
/*     record read is written earlier in the same call.                       */
/*   - The first call on a device looks the array's address up (no allocation);*/
/*     make that call before a stream capture begins.                          */
/* ------------------------------------------------------------------------- */
#define MASSV_SPEC_ACCEPT_STATIC_BYTES (4u << 20)
size_t massv_spec_accept_static_limit(void);      /* = MASSV_SPEC_ACCEPT_STATIC_BYTES */
int massv_spec_accept_static(const float* target_logits, const float* draft_logits,
                             const int32_t* draft_tokens, const float* uniforms,
                             float temperature, int32_t B, int32_t gamma, int32_t V,
                             int32_t* n_accepted, int32_t* out_tokens, void* stream);

/* ------------------------------------------------------------------------- */
/* lm_head_greedy_accept: massv_lm_head_logits followed by massv_spec_accept   */
/* at temperature 0 (Section 2.1: a draft is kept iff it is the arg-max of the */
/* target's distribution at its position), without writing the logits: the     */
/* projection keeps per row only the largest logit and its lowest column.      */
/* Results are identical to the two calls.                                     */
/* x [B][gamma+1][H] (dtype); final_norm [H] or NULL; w_lm [V][H] in streaming */
/* layout; draft_tokens [B][gamma] int32 (NULL iff gamma == 0); n_accepted [B],*/
/* out_tokens [B][gamma+1] int32 out.  bf16 only, limits as for the two calls. */
/* ------------------------------------------------------------------------- */
size_t massv_lm_head_greedy_accept_workspace(int32_t B, int32_t gamma, int32_t H, int32_t V, int32_t dtype);
int massv_lm_head_greedy_accept(const void* x, const void* final_norm, const void* w_lm,
                                const int32_t* draft_tokens, int32_t B, int32_t gamma, int32_t H, int32_t V,
                                float norm_eps, int32_t dtype, int32_t* n_accepted, int32_t* out_tokens,
                                void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- */
/* lm_head_accept: massv_lm_head_logits followed by massv_spec_accept at any   */
/* temperature, in one call (Section 2.1: the scores p_i and the accept rule). */
/* T = 0 is massv_lm_head_greedy_accept (no logits are written; `logits` may   */
/* be NULL).  T > 0: the logits ARE written to `logits` -- the rule reads      */
/* p_i(x_i) from them and re-reads one row per sequence for the final draw --  */
/* but the projection also leaves, per row and per piece of the vocabulary,    */
/* the piece's largest logit, its column and its sum of exp((x - largest)/T),  */
/* so the accept rule's first pass streams the draft rows only.  Results equal */
/* those of the two separate calls wherever no decision lies within rounding   */
/* (the row sums are formed from differently cut pieces: agreement to ~1e-7).  */
/* Arguments as for the two calls; x [B][gamma+1][H] (dtype), logits           */
/* [B*(gamma+1)][V] float32 out.  bf16 only.                                   */
/* ------------------------------------------------------------------------- */
size_t massv_lm_head_accept_workspace(int32_t B, int32_t gamma, int32_t H, int32_t V, int32_t dtype);
int massv_lm_head_accept(const void* x, const void* final_norm, const void* w_lm,
                         const float* draft_logits, const int32_t* draft_tokens, const float* uniforms,
                         float temperature, int32_t B, int32_t gamma, int32_t H, int32_t V,
                         float norm_eps, int32_t dtype, float* logits, int32_t* n_accepted, int32_t* out_tokens,
                         void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- */
/* commit_tokens: bookkeeping after spec_accept, on the device so that the     */
/* decoding loop of Section 2.1 needs no host round trip: sequence b keeps its */
/* n_b accepted drafts and the final token, so                                 */
/*   last_token[b] = out_tokens[b][n_accepted[b]]   (input of the next step)   */
/*   kv_len[b]    += n_accepted[b] + 1              (cache rows now valid)     */
/* Rows written for rejected drafts stay in the caches beyond the new kv_len   */
/* and are overwritten by the next step: nothing is moved.                     */
/* n_accepted [B], out_tokens [B][gamma+1] int32 in; kv_len [B] int32 in/out;  */
/* last_token [B] int32 out (may be NULL); all device pointers.                */
/* ------------------------------------------------------------------------- */
int massv_commit_tokens(const int32_t* n_accepted, const int32_t* out_tokens, int32_t* kv_len,
                        int32_t* last_token, int32_t B, int32_t gamma, void* stream);

/* ------------------------------------------------------------------------- */
/* spec_tvd: total variation distance of Section 6 between the target and the */
/* draft distribution of every row, TVD = 1/2 sum_x |p(x) - q(x)| with         */
/* p = softmax(target_logits[r]/T), q = softmax(draft_logits[r]/T); 1 - TVD is */
/* the expected acceptance probability of a token drawn from q at that row.   */
/* ------------------------------------------------------------------------- */
size_t massv_spec_tvd_workspace(int32_t rows, int32_t V);

/* target_logits, draft_logits [rows][V] float32 in (device); temperature > 0, finite;
 * tvd [rows] float64 out (device), absolute error below 1e-6 (exponentials in float, sums in double).
 * rows <= 32767.  Logits as for massv_spec_accept. */
int massv_spec_tvd(const float* target_logits, const float* draft_logits, float temperature,
                   int32_t rows, int32_t V, double* tvd,
                   void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- */
/* embed_tokens: x[m, :] = table[tokens[m], :], the input of the first layer   */
/* for the tokens a drafting or verify step feeds back (Section 2.1's loop).   */
/* table [V][H] and x [M][H] of `dtype`, row-major, device; tokens [M] int32   */
/* device.  A token outside [0,V) gives a row of zeros.  H * elem size must be */
/* a multiple of 4 bytes.                                                      */
/* ------------------------------------------------------------------------- */
int massv_embed_tokens(const void* table, const int32_t* tokens, void* x,
                       int32_t M, int32_t H, int32_t V, int32_t dtype, void* stream);

/* ------------------------------------------------------------------------- */
/* linear: Y = act(X W^T + bias) for prefill-sized inputs, the compute-bound   */
/* counterpart of the verify projections.  Section 3.1: the drafter's          */
/* multimodal projector g_psi maps each of the m vision features (dimension    */
/* d_vis) to the language model's embedding dimension; it has the target       */
/* projector's architecture, a small MLP, i.e. a few calls of this entry point */
/* over M = (images x m) rows.  The same call serves the projections of an     */
/* image-token prefill.                                                        */
/* ------------------------------------------------------------------------- */
typedef enum { MASSV_LIN_NONE = 0, MASSV_LIN_SILU = 1, MASSV_LIN_GELU_TANH = 2, MASSV_LIN_GELU_ERF = 3 } massv_linear_act;

size_t massv_linear_workspace(int32_t M, int32_t N, int32_t K, int32_t dtype);

/* x [M][K] row-major (dtype) in; w [N][K] (dtype) in the streaming layout of massv_weight_pack;
 * bias [N] (dtype) or NULL; y [M][N] row-major (dtype) out; all device pointers.  fp32 accumulation, one
 * rounding to dtype after the activation.  bf16 only; K % 64 == 0 and N % 16 == 0, any M >= 1, else
 * MASSV_EUNSUPPORTED.  The workspace receives X in operand order. */
int massv_linear(const void* x, const void* w, const void* bias, void* y, int32_t M, int32_t N, int32_t K,
                 int32_t act, int32_t dtype, void* workspace, size_t workspace_bytes, void* stream);

/* The same with two optional row-major [M][N] operands applied after the activation, in this order:
 *   Y = act(X W^T + bias) * mul + add
 * mul (or NULL): e.g. the up projection's rows, for the gated MLP act(gate(x)) * up(x); add (or NULL): e.g. the
 * residual stream.  add may be y itself (each element is read before it is written); mul and x must not overlap y. */
int massv_linear_ex(const void* x, const void* w, const void* bias, const void* mul, const void* add, void* y,
                    int32_t M, int32_t N, int32_t K, int32_t act, int32_t dtype, void* workspace,
                    size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- */
/* rmsnorm: y[m, :] = x[m, :] * gain / sqrt(mean(x[m, :]^2) + eps) for any     */
/* number of rows (the norm of a prompt pass; inside the verify step the norms */
/* are fused into the neighbouring kernels).  x, y [M][H] row-major, gain [H], */
/* all of `dtype`, device; y must not overlap x.  Sums in fp32.                */
/* ------------------------------------------------------------------------- */
int massv_rmsnorm(const void* x, const void* gain, void* y, int32_t M, int32_t H, float eps, int32_t dtype,
                  void* stream);

/* ------------------------------------------------------------------------- */
/* Timing hook (diagnostic; for callers that want one kernel's duration        */
/* without a profiler).  Arms a one-shot request on the CALLING THREAD: the    */
/* next launch of kernel `kernel_id` made by a library call from this thread   */
/* is issued with hipExtLaunchKernelGGL(start_event, stop_event), so the two   */
/* events carry that kernel's own begin and end timestamps; the request is     */
/* then gone.  Events are hipEvent_t created by the caller with timing         */
/* enabled; the caller synchronises and reads hipEventElapsedTime.             */
/* kernel_id < 0 disarms.                                                      */
/* Do not arm while the stream is being captured into a graph.                 */
/* ------------------------------------------------------------------------- */
typedef enum {
    MASSV_K_QKV = 0,          /* fused q/k/v projection of verify_layer */
    MASSV_K_ATTENTION = 1,    /* the split-KV attention kernel */
    MASSV_K_ATTN_COMBINE = 2, /* merge of the KV splits */
    MASSV_K_OPROJ = 3,        /* output projection + residual */
    MASSV_K_GATEUP = 4,       /* gate/up projection + activation */
    MASSV_K_DOWN = 5,         /* down projection + residual */
    MASSV_K_LMHEAD = 6,       /* vocabulary projection of lm_head_logits */
    MASSV_K_ACCEPT_STATS = 7, /* pass 1 of spec_accept over all logit rows */
    MASSV_K_RESIDUAL_MASS = 8,/* pass 2 of spec_accept over the resampled rows */
    MASSV_K_LINEAR = 9,       /* the tile kernel of massv_linear */
    MASSV_K_PREFILL_ATTENTION = 10  /* the bf16 kernel of prefill_attention */
} massv_kernel_id;

int massv_trace_kernel(int kernel_id, void* start_event, void* stop_event);

#ifdef __cplusplus
}
#endif
#endif /* MASSV_VERIFY_H */
