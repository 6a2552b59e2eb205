/*
 * qspec.h — C ABI of the dual-mode W4 linear layer of QSpec (arXiv 2410.11305)
 * for AMD MI355X (gfx950).
 *
 * One packed 4-bit weight tensor serves two activation modes (paper Sec. 3:
 * only the activation scheme is switched, no second copy of the weights):
 *   draft  (W4A4):  qspec_quant_act  ->  qspec_gemm_w4a4
 *   verify (W4A16): qspec_gemm_w4a16
 * Quantisation is group-wise along the input dimension K with group size 128
 * (paper Sec. 4.1, "Implementations").
 *
 * Notation: x fp16 [M,K] row-major (tokens x in-features); the weight is
 * [N,K] (out x in), y = x W^T is fp16 [M,N] row-major; G = K/128.
 *
 * Conventions shared by every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller, 16-byte aligned.
 *     The library allocates nothing and keeps no state between calls (but see
 *     the workspace rule below).
 *   - `stream` is a hipStream_t (NULL = the default stream).  All work is
 *     enqueued on it; the call returns without synchronising.
 *   - The return value is a qspec_status.  Arguments are validated on the
 *     host first; on any error nothing is launched.  No exception or abort
 *     crosses this boundary.
 *   - Shapes: group must be 128, K a positive multiple of 128, N a positive
 *     multiple of 16, M >= 1.  Anything else is QSPEC_ERR_SHAPE.
 *   - Input and output ranges must not overlap.
 *   - Non-finite activations: behaviour unspecified.
 *
 * Packed weight blob (written by qspec_pack_weights, N*K/2 + N*G*2 bytes)
 *   codes  : tiles of 16 output rows x 128 input features (one group), 1024
 *            bytes each, tile (T = n/16, g = k/128) at byte (T*G + g)*1024.
 *            Inside a tile the 16 bytes at offset 16*(16*kb + n%16), kb = 0..3,
 *            are four 32-bit little-endian words of row n; word i (i = 0..3)
 *            holds the 8 codes k%128 in [32*i + 8*kb, 32*i + 8*kb + 8).  In a
 *            word the eight 4-bit two's-complement codes c0..c7 sit at bit
 *            positions 4*p with p = 0..7 holding c0,c2,c4,c6,c1,c3,c5,c7.
 *   scales : fp16, transposed to [G][N], starting at byte N*K/2.
 *
 * Quantised activations (written by qspec_quant_act)
 *   qa : M rows of K/2 bytes, 64 bytes per group.  Each aligned run of 8
 *        codes is one 32-bit word with the nibble order of a weight word
 *        (c0,c2,c4,c6,c1,c3,c5,c7 from bit 0 upward); inside a group the word
 *        of codes [32*i + 8*kb, +8) is stored at word position 4*kb + i.
 *   sa : fp32 [M][G], row-major.
 */
#ifndef QSPEC_H
#define QSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  QSPEC_OK = 0,
  QSPEC_ERR_NULL = 1,        /* a required pointer is NULL                    */
  QSPEC_ERR_SHAPE = 2,       /* M, N, K or group outside what is supported    */
  QSPEC_ERR_ALIGN = 3,       /* a pointer is not 16-byte aligned              */
  QSPEC_ERR_WORKSPACE = 4,   /* workspace smaller than qspec_workspace_bytes  */
  QSPEC_ERR_HIP = 5,         /* the HIP runtime refused the launch            */
  QSPEC_ERR_UNSUPPORTED = 6  /* not gfx950; a forced plan has no kernel; a shape outside what a variant entry point takes */
} qspec_status;

/* Human-readable name of a status code (static storage, never NULL). */
const char* qspec_status_string(int status);

/* Library version: 1000*major + minor. */
int qspec_version(void);

/* Size in bytes of the packed blob for an [N,K] weight; 0 if the shape is not
 * supported. */
size_t qspec_packed_weight_bytes(int N, int K, int group);

/* Scratch the GEMM entry points need for an (M,N,K) problem (partial sums of
 * K-slices that several workgroups produce); 0 when none is needed.  Returns 0
 * for unsupported shapes as well (the GEMM call reports those).
 * Workspace rule: the first 16 KiB of a workspace hold arrival counters.  They
 * must be ZERO when the first GEMM call that uses the workspace is enqueued;
 * every GEMM call leaves them zero again, so one zero-filled allocation serves
 * any number of calls in turn.  The rest is scratch with no meaning between
 * calls.  Two GEMM calls that may run at the same time (different streams) need
 * a workspace each. */
size_t qspec_workspace_bytes(int M, int N, int K, int group);

/*
 * Build the shared weight blob (paper Sec. 3: one weight tensor for both
 * modes; Sec. 4.1: group size 128).  Runs once per layer, off the token path.
 *   codes      int8 [N,K] row-major, values in [-8,7]; only the low 4 bits of
 *              each value are stored, out-of-range input is not detected.
 *   scales_f16 fp16 [N,G] row-major; weight value = code * scale.
 *   packed     out, qspec_packed_weight_bytes(N,K,group) bytes.
 */
int qspec_pack_weights(const int8_t* codes, const void* scales_f16, int N, int K, int group,
                       void* packed, void* stream);

/* Inverse of qspec_pack_weights (debug / round-trip check): recovers the
 * canonical int8 [N,K] codes and fp16 [N,G] scales from a blob. */
int qspec_unpack_weights(const void* packed, int N, int K, int group,
                         int8_t* codes, void* scales_f16, void* stream);

/*
 * Activation quantiser of the draft mode (paper Sec. 1: in W4A4 activations
 * are 4-bit as well).  Per token m and group j, in binary32:
 *   a = max|x|, s = a / 7 (IEEE division), q = clamp(rne(x / s), -8, 7)
 * (IEEE division, round half to even); an all-zero group gives s = 0, q = 0.
 *   x_f16 fp16 [M,K];  qa out, M*K/2 bytes;  sa out, fp32 [M,G].
 */
int qspec_quant_act(const void* x_f16, int M, int K, int group,
                    uint8_t* qa, float* sa, void* stream);

/*
 * Producers of draft-mode activations fused with the quantiser (paper Sec. 3.1,
 * draft phase: every linear layer of the draft pass consumes 4-bit activations
 * quantised on the fly; in a Llama-shaped block, Sec. 4.1, those activations
 * come out of an RMSNorm or of SiLU(gate) * up).  One launch writes what
 * qspec_quant_act would write for the fp16 tensor h the producer computes:
 *   qspec_rmsnorm_quant:   r = fp32(1 / sqrt(sum_k x[m,k]^2 / K + eps))  (binary64 inside)
 *                          h[m,k] = fp16(fp32((x[m,k] * w[k]) * r))
 *   qspec_silu_mul_quant:  s = fp32(g / (1 + exp(-g)))                  (binary64 inside)
 *                          h[m,i] = fp16(fp32(s * u)),  g = gate_up[m,i], u = gate_up[m,I+i]
 *   x_f16       fp16 [M,K];  weight_f16 fp16 [K];  eps >= 0, finite (an all-zero row with
 *               eps = 0 gives zeros);
 *   gate_up_f16 fp16 [M,2I], the gate in the first I columns; I a positive multiple of 128;
 *   qa, sa      out, as qspec_quant_act writes them for h ([M,K] resp. [M,I]);
 *   rotate      flag bits.  Bit 0 (value 1): h is replaced by its rotation
 *               (qspec_hadamard_quant below, applied to the fp16 tensor h) before it is
 *               stored and quantised.  Bit 1 (value 2): the codes are stored in the widened
 *               format of qspec_quant_act_wide (qa then holds M*K resp. M*I bytes), for a
 *               consumer that runs qspec_gemm_w4a4_wide.  Other bits: QSPEC_ERR_SHAPE;
 *   h_f16       out, fp16 [M,K] resp. [M,I], or NULL when the tensor itself is not
 *               needed (the draft pass needs only the codes).
 */
int qspec_rmsnorm_quant(const void* x_f16, const void* weight_f16, float eps, int M, int K, int group,
                        int rotate, uint8_t* qa, float* sa, void* h_f16, void* stream);
int qspec_silu_mul_quant(const void* gate_up_f16, int M, int I, int group,
                         int rotate, uint8_t* qa, float* sa, void* h_f16, void* stream);

/*
 * Outlier-spreading rotation fused with the quantiser (paper Sec. 4.1 builds on
 * existing 4-bit quantisers, a rotation-based one among them; the paper gives no
 * detail, the block-diagonal form is this library's): every group of 128 input
 * features is multiplied by the Sylvester Hadamard matrix H_128 (natural order,
 * H[i][j] = (-1)^popcount(i & j)) and by 2^-3, then quantised as qspec_quant_act does:
 *   h[m, 128 j .. 128 j + 127] = fp16( x[m, 128 j .. 128 j + 127] H_128 / 8 )
 * The transform runs in binary32 as the fast transform with stages h = 1, 2, ..., 64
 * (stage h replaces v[i], v[i+h] by v[i] + v[i+h], v[i] - v[i+h]).  A layer that is
 * fed these activations holds its weights in the rotated basis (w_g H_128 / 16 per
 * group, prepared offline before qspec_pack_weights), so that h w'^T = x w^T; the
 * verify mode takes h_f16 as its input.
 *   x_f16 fp16 [M,K];  qa, sa out, as qspec_quant_act writes them for h;
 *   h_f16 out, fp16 [M,K], or NULL.
 */
int qspec_hadamard_quant(const void* x_f16, int M, int K, int group,
                         uint8_t* qa, float* sa, void* h_f16, void* stream);

/*
 * Reordering activation quantiser (paper Sec. 4.1 builds on existing 4-bit quantisers,
 * one of which moves the few large channels together and keeps them in higher
 * precision; the paper gives no detail, this form is this library's and needs no
 * mixed-precision GEMM).  Position p of the reordered row takes channel perm[p]; the
 * last n_outlier_groups groups of the reordered row are quantised to 239 levels,
 *   a = max|x|, s = a / 119, q8 = clamp(rne(x / s), -119, 119)   (binary32, IEEE division)
 * and written as two 4-bit groups, q8 = 16 hi + lo with lo in [-8,7], hi in [-7,7],
 * with scales 16 s and s; all other groups as qspec_quant_act does.  Output: G' = G +
 * n_outlier_groups groups (K' = 128 G'): the ordinary groups in order, then hi, lo of
 * each outlier group.  The weights of the layer hold their columns in the same order,
 * each outlier group twice in a row (prepared offline, before qspec_pack_weights with
 * K'); qspec_gemm_w4a4 is then called with K'.
 *   x_f16    fp16 [M,K];  perm  int32 [K], 16-byte aligned, a permutation of 0..K-1
 *            (not checked; entries outside [0,K) are clamped);
 *   0 <= n_outlier_groups <= K/128;
 *   qa  out, M*K'/2 bytes;  sa  out, fp32 [M,G'];
 *   h_f16    out, fp16 [M,K'] or NULL: the reordered row with a zero group after each
 *            outlier group, i.e. the verify-mode input for the same weights.
 */
int qspec_reorder_quant(const void* x_f16, const int32_t* perm, int M, int K, int group,
                        int n_outlier_groups, uint8_t* qa, float* sa, void* h_f16, void* stream);

/*
 * Draft-mode product (paper Sec. 1: W4A4 runs on the low-precision matrix
 * units without dequantising to a higher precision):
 *   P[m,n,j] = sum_{k in group j} qa[m,k] * qw[n,k]             (int32, exact)
 *   y[m,n]   = fp16( sum_j float(P[m,n,j]) * sa[m,j] * sw[n,j] ) (fp32 sums)
 *   packed  blob from qspec_pack_weights for the same (N,K);
 *   qa, sa  from qspec_quant_act for the same (M,K);
 *   y_f16   out, fp16 [M,N];
 *   workspace  at least qspec_workspace_bytes(M,N,K,group) bytes (may be NULL
 *              when that is 0); see the workspace rule at qspec_workspace_bytes.
 */
int qspec_gemm_w4a4(const void* packed, const uint8_t* qa, const float* sa,
                    int M, int N, int K, int group,
                    void* y_f16, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same quantiser and the same draft-mode product (paper Sec. 1, W4A4; Sec. 4.1,
 * groups of 128) with the activation codes kept in a second device format for the shapes
 * whose product runs on the tiled kernel (more than 64 tokens, or 48 on very wide layers):
 * every code in a byte of its own, as int8 16 * code, 128 bytes per token row and group in
 * the order of that kernel's LDS rows (byte b of the packed group's 64 bytes gives byte b
 * = 16 * its low-nibble code and byte 64 + b = 16 * its high-nibble code).  The kernel then
 * takes the codes global -> LDS directly instead of widening them in registers.  Codes and
 * scales are those of qspec_quant_act bit for bit; only the storage differs.
 *   qspec_w4a4_takes_wide   1 if qspec_gemm_w4a4_wide accepts this shape, else 0 (also 0
 *                           for a shape the library refuses);
 *   qspec_quant_act_wide    x_f16 fp16 [M,K];  qa8 out, M*K bytes;  sa out, fp32 [M,G];
 *   qspec_gemm_w4a4_wide    arguments as qspec_gemm_w4a4 with qa8 in place of qa;
 *                           QSPEC_ERR_UNSUPPORTED (nothing launched) for a shape whose
 *                           product runs on a kernel that reads packed codes.
 */
int qspec_w4a4_takes_wide(int M, int N, int K, int group);
int qspec_quant_act_wide(const void* x_f16, int M, int K, int group,
                         int8_t* qa8, float* sa, void* stream);
int qspec_gemm_w4a4_wide(const void* packed, const int8_t* qa8, const float* sa,
                         int M, int N, int K, int group,
                         void* y_f16, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Verify-mode product (paper Sec. 1: W4A16 dequantises the 4-bit weights to
 * fp16 at run time and multiplies with fp16 activations):
 *   y[m,n] = fp16( sum_k x[m,k] * qw[n,k] * sw[n, k/128] )       (fp32 sums)
 *   x_f16 fp16 [M,K]; other arguments as for qspec_gemm_w4a4.
 */
int qspec_gemm_w4a16(const void* packed, const void* x_f16,
                     int M, int N, int K, int group,
                     void* y_f16, void* workspace, size_t workspace_bytes, void* stream);

/*
 * qspec_gemm_w4a16 for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, result and kernels as qspec_gemm_w4a16, but the
 * K-slice scratch (arrival counters and partial sums) is a fixed array inside the
 * library's device image, 32 MiB + 16 KiB per GPU, held by every
 * GPU the library runs on until the process ends.  The call allocates nothing.
 *   - A shape whose plan needs more than that returns QSPEC_ERR_WORKSPACE and launches
 *     nothing (qspec_workspace_bytes tells: use qspec_gemm_w4a16 with a workspace).
 *   - Every call on one GPU shares that GPU's array; the counters are cleared by a small
 *     kernel in front of the GEMM.  Calls that may overlap on one GPU (different
 *     streams) race: serialise them, or give all but one a workspace of their own.
 *   - The first call on a device looks up the array's device address
 *     (hipGetSymbolAddress); make that first call outside graph capture.
 */
int qspec_gemm_w4a16_noalloc(const void* packed, const void* x_f16,
                             int M, int N, int K, int group,
                             void* y_f16, void* stream);

/*
 * The MLP of a decoder block in the draft pass as ONE persistent launch (paper Sec. 3.1,
 * draft phase: every linear layer of the draft pass runs in W4A4 on activations quantised
 * on the fly; Sec. 3.2: the method's gain rests on a fast draft pass):
 *   gate_up = W4A4( qa_h, sa_h ; packed_gate_up )            fp16 [M, 2I], gate first
 *   (qa_i, sa_i) = what qspec_silu_mul_quant writes for gate_up (rotate = 0)
 *   y = W4A4( qa_i, sa_i ; packed_down )                     fp16 [M, H]
 * i.e. exactly qspec_gemm_w4a4, qspec_silu_mul_quant, qspec_gemm_w4a4 in a row, for
 * 1 <= M <= 32 tokens.
 *   packed_gate_up  blob of the [2I, H] gate/up weight;  packed_down  blob of the [H, I] weight;
 *   qa_h, sa_h      quantised block input for K = H (qspec_rmsnorm_quant / qspec_quant_act);
 *   gate_up_f16, qa_i, sa_i, y_f16   outputs (the first three are also how the stages talk);
 *   workspace       qspec_mlp_draft_workspace_bytes(...) bytes of counters, ZERO before the
 *                   first use; every successful call leaves them zero;
 *   status_word     device int32 the caller set to 0.  The launch is one workgroup per
 *                   compute unit and needs all of them resident together (an otherwise idle
 *                   GPU).  A workgroup that has waited for the others longer than a bounded
 *                   number of polls (about 0.1 s) writes 1 there and exits; y_f16 is then
 *                   invalid and the workspace must be zeroed again.  Every kernel exits.
 * Returns QSPEC_ERR_UNSUPPORTED for shapes outside the kernel (M > 32; more than 6 gate/up
 * or 2 down tiles of 16 outputs per compute unit; more than 96 KB of down-projection
 * weights per compute unit, e.g. I > 12288 with H <= 4096): use the separate calls.
 */
size_t qspec_mlp_draft_workspace_bytes(int M, int H, int I, int group);
int qspec_mlp_draft(const void* packed_gate_up, const void* packed_down,
                    const uint8_t* qa_h, const float* sa_h, int M, int H, int I, int group,
                    void* gate_up_f16, uint8_t* qa_i, float* sa_i, void* y_f16,
                    void* workspace, size_t workspace_bytes, int* status_word, void* stream);

/*
 * Debug entry: the exact per-group integer partial sums of the draft product
 * for output columns n0 .. n0+n_count-1 (n0 and n_count multiples of 16):
 *   partials[m, n - n0, j] = P[m,n,j], int32 [M, n_count, G] row-major.
 */
int qspec_gemm_w4a4_partials(const void* packed, const uint8_t* qa,
                             int M, int N, int K, int group,
                             int n0, int n_count, int32_t* partials, void* stream);

/*
 * Greedy acceptance after the verify pass (paper Sec. 3.1, "Verify Phase" and
 * "Acceptance Policy").  The verify pass takes, per sequence, the last committed
 * token followed by the gamma drafted tokens and returns gamma + 1 rows of
 * logits; row j is the distribution of the token after input j.  Draft j
 * (0-based) is accepted exactly when every earlier draft was accepted and it
 * equals the top-1 token of row j; the first rejection discards the later
 * drafts.  The token emitted after the accepted ones is the top-1 of the row
 * where the walk stopped (the corrected token, or one extra token when all
 * gamma drafts were accepted).  Top-1 under ties: the lowest token id; -0 and
 * +0 are equal.  NaN logits: behaviour unspecified.
 *   logits_f16    fp16 [B, gamma+1, V] row-major, 16-byte aligned;
 *   draft_tokens  int32 [B, gamma];
 *   n_accept      out, int32 [B], number of accepted drafts (0..gamma);
 *   out_tokens    out, int32 [B, gamma+1]: the accepted drafts, then the emitted
 *                 token, then -1;
 *   workspace     at least qspec_accept_workspace_bytes(B, gamma, V) bytes of
 *                 scratch, 16-byte aligned, contents meaningless before and after
 *                 (nothing to clear, no counters).
 * int32 arrays need 4-byte alignment only.  B >= 1, gamma >= 1, V >= 1,
 * B*(gamma+1) <= 65535; otherwise QSPEC_ERR_SHAPE.
 */
size_t qspec_accept_workspace_bytes(int B, int gamma, int V);
int qspec_greedy_accept(const void* logits_f16, const int32_t* draft_tokens, int B, int gamma, int V,
                        int32_t* n_accept, int32_t* out_tokens,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * KV-cache overwrite (paper Sec. 3.1, "KV Cache Overwriting"): the cache entries
 * of the accepted tokens are replaced by the ones the verify pass computed.
 * For every sequence b, rows 0 .. n_accept[b] of kv_verify (row 0 belongs to the
 * last committed token, row j >= 1 to draft j-1) are copied to cache rows
 * pos[b] .. pos[b] + n_accept[b]; rows after the first rejection are not
 * copied, target rows outside [0, S) are skipped, n_accept is clamped to
 * [0, gamma].  Call it once for K and once for V (or once for a fused layout).
 *   kv_verify_f16 fp16 [B, gamma+1, D];  cache_f16 in/out, fp16 [B, S, D];
 *   n_accept, pos int32 [B] (device memory; n_accept as written by
 *   qspec_greedy_accept);  D a positive multiple of 8.
 */
int qspec_kv_overwrite(const void* kv_verify_f16, const int32_t* n_accept, const int32_t* pos,
                       int B, int gamma, int D, int S, void* cache_f16, void* stream);

/*
 * Debug entry (benchmark A/B and tests): force the kernel plan the GEMM entry points
 * and qspec_workspace_bytes use, instead of the library's own choice.  `name` is one of
 *   "QSPEC_KERNEL"            value "generic": untiled reference kernels for M > 32
 *   "QSPEC_STREAM_W4A4",  "QSPEC_STREAM_W4A16"   value "NT,S" or "NT,S,MS": tiles per
 *                             workgroup, K-slices, token-row blocks of the streaming kernels
 *   "QSPEC_STREAM_MAX_W4A4"   largest M the draft-mode streaming kernel takes (32..128)
 *   "QSPEC_TILE_W4A4",    "QSPEC_TILE_W4A16"     value "shape,S": workgroup shape, K-slices
 *   "QSPEC_MLP_SPIN"          polls before a workgroup of qspec_mlp_draft gives up waiting
 * `value` NULL (or unparsable) clears that override; both are host strings.  The same
 * names are read from the environment once, at the library's first use; no entry point
 * reads the environment afterwards.  A forced plan that names no existing kernel instance
 * falls back to the library's choice or makes the GEMM call return
 * QSPEC_ERR_UNSUPPORTED.  Process-wide state: do not call it while another thread is
 * inside a GEMM entry point.  Returns QSPEC_ERR_SHAPE for an unknown name.
 */
int qspec_debug_set_plan(const char* name, const char* value);

/*
 * Debug entry: name of the device kernel the GEMM entry points select for an
 * (M,N,K) problem, e.g. "gemm_stream_kernel<false, 2, 3>" (mode 0 = W4A16
 * verify, 1 = W4A4 draft).  It matches the symbol a profiler reports, so that
 * benchmark timings can be set beside profiler output.  Writes a NUL-terminated
 * string of at most cap-1 characters to `out` (host memory); returns a status.
 */
int qspec_describe_kernel(int mode_w4a4, int M, int N, int K, int group, char* out, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* QSPEC_H */
