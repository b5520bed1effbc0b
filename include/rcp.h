/*
 * rcp.h - C ABI of the MI355X (gfx950) W2A4 look-up-table GEMV path of RCP
 * ("Rotate, Clip, and Partition", arXiv 2502.15779).
 *
 * The library implements the decode-time linear layer of the paper's Section 4.4
 * ("Look-up Table (LUT) Inference for Non-uniform W2A4 GEMV") and the two steps
 * that feed it:
 *
 *   rcp_pack_weights      offline export: LDP thresholds -> 2-bit indices, and the
 *                         per-output-channel 4-entry dequantisation LUT
 *                         (Section 4.3, Eqns. for p_i / t_i / Q_LDP / w_i, and the
 *                         LUT equation of Section 4.4)
 *   rcp_rotate_quant_act  online Hadamard rotation (Appendix, definition of the
 *                         normalised Hadamard matrix; Section 2.1 for where online
 *                         rotations sit) + per-token symmetric int4 quantisation
 *                         (Appendix table "Quantization configurations")
 *   rcp_w2a4_gemv         O = S * sum_k LUT[h][W_q[h][k]] * X_q[k]  (Section 4.4,
 *                         "Fast GEMV via Latency Hiding": tensor list and shapes)
 *
 * General rules
 *   - Every pointer named below is a DEVICE pointer unless it is marked "host".
 *     All device buffers are owned by the caller; the library allocates nothing
 *     that outlives a call and frees nothing the caller passed in.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). Work
 *     is enqueued on it and the call returns without synchronising.
 *   - Return value: RCP_OK (0) or a negative rcp_status. On error nothing has
 *     been enqueued and no output byte has been written; rcp_last_error() holds
 *     a message.
 *   - Device buffers must be 16-byte aligned (anything a GPU allocator returns).
 *
 * Shapes and names: the weight matrix is N (output channels, the paper's H) by
 * K (input channels, the paper's C). M is the number of tokens (1 for GEMV).
 *
 * ---------------------------------------------------------------------------
 * Data layouts
 *
 * Packed weight indices ("W_q"), N*K/4 bytes.  The paper stores four 2-bit
 * indices per byte in row-major order; this library stores the same N*K 2-bit
 * indices as bit planes so that a CDNA4 lane can feed them to the packed-int4
 * dot instruction without per-weight shifts:
 *   - rows are grouped four at a time: g = h / 4, r = h % 4
 *   - columns eight at a time:         o = k / 8, j = k % 8
 *   - a "cell" (g, o) is two little-endian uint32 words (B0, B1), 8 bytes, stored
 *     at byte offset 8 * (g * (K/8) + o)
 *   - bit (4*j + r) of B0 is bit 0 of idx[4g+r][8o+j]; the same bit of B1 is
 *     bit 1 of that index.  (idx = 0..3 selects the LUT entry.)
 *
 * LUT / codebook ("W-hat"): fp16 [N][4], entry l of row h at half-word 4*h + l,
 * ascending in l.
 *
 * Quantised activation ("X_q"): M * K/2 bytes; token m starts at byte m*K/2.
 * Byte b holds q[2b] in its low nibble and q[2b+1] in its high nibble, each a
 * two's-complement int4 in [-8, 7].  Scale ("S"): fp16 [M].
 *
 * Output ("O"): row-major M x N, fp16 or fp32.
 * Partial sums (verification output): int32 [M][N][4],
 *   P[m][h][l] = sum over k with idx[h][k] == l of q[m][k].
 *
 * Group-wise quantisation units (the *_grouped calls; the paper's deployed setting,
 * Appendix table "Quantization configurations": weight group size 128).  Columns
 * 128g .. 128g+127 of a row form group g, NG = K/128 groups per row; every (row, group)
 * has its own clip range, partition fractions and four levels.
 *   Grouped packed indices, N*K/4 bytes: the same 8-byte cells, a "unit" being the two
 *   cells of 16 consecutive columns (16 bytes).  The K/16 units of a group of four rows
 *   g4 = h/4 start at byte g4 * (K/16) * 16 and are ordered so that the lanes of a
 *   wavefront that each own one quantisation group read consecutive units: group g
 *   belongs to round g/32 and lane g%32, a round holds R = min(32, NG - 32*(g/32))
 *   groups, and unit i (0..7: columns 128g + 16i .. 128g + 16i + 15) of group g sits at
 *   unit position 256*(g/32) + i*R + g%32.  Inside a unit the cell of the lower eight
 *   columns comes first.
 *   Grouped LUT: fp16 [N/4][NG][4 rows][4 levels]: level l of row h, group g at half-word
 *   (((h/4)*NG + g)*4 + h%4)*4 + l.  N*NG*8 bytes.
 *   Grouped partial sums: int32 [N][NG][4].
 *
 * 3-bit variant (the *_w3 calls; Section 4.3, paragraph on the asymmetric normal-float
 * 3-bit format): eight levels per output channel, idx = b0 + 2*b1 + 4*b2.
 *   3-bit packed indices, 3*N*K/8 bytes: three bit planes.  A group of four rows g4 = h/4 is
 *   K/32 "units" of 4 rows x 32 columns and starts at byte g4 * (K/32) * 48.  Units go in
 *   blocks of 64 (block j = u/64 starts 3072*j bytes into the row group); a block of
 *   R = min(64, K/32 - 64*j) units stores plane 0 of its R units, then plane 1, then plane
 *   2, so that the 64 lanes of a wavefront read each plane as one contiguous run: plane p
 *   of unit u lies 16*R*p + 16*(u%64) bytes into its block.  Those 16 bytes are four
 *   little-endian uint32 words; word (k%32)/8 covers eight columns, and its bit
 *   4*(k%8) + h%4 is bit p of idx[h][k].
 *   3-bit LUT: fp16 [N][8], ascending.  3-bit partial sums: int32 [N][8].
 */
#ifndef RCP_H
#define RCP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RCP_OK = 0,
    RCP_ERR_NULL = -1,        /* a required pointer is NULL                         */
    RCP_ERR_SHAPE = -2,       /* N, K, M out of range or not a supported multiple   */
    RCP_ERR_ALIGN = -3,       /* a device buffer is not 16-byte aligned             */
    RCP_ERR_UNSUPPORTED = -4, /* dtype / rotation / M outside the compiled set      */
    RCP_ERR_WORKSPACE = -5,   /* workspace missing or too small                     */
    RCP_ERR_HIP = -6          /* the HIP runtime reported an error (see last error) */
} rcp_status;

typedef enum { RCP_F16 = 0, RCP_F32 = 1, RCP_BF16 = 2 } rcp_dtype;

typedef enum {
    RCP_ROT_NONE = 0, /* y = x (the rotation was fused into the weights offline)   */
    RCP_ROT_WHT = 1,  /* y = H_K x, K a power of two                               */
    RCP_ROT_KRON = 2, /* y = (H_{n_wht} (x) Q) x, K = n_wht * m                    */
    RCP_ROT_HEADS = 3 /* y = (H_{n_wht} (x) I_m) x: Hadamard across n_wht heads of m channels (the online
                         rotation of the self-attention output before the out-projection, Section 2.1);
                         2 <= n_wht <= 64, m a multiple of 8, K <= RCP_MAX_WHT; Q is ignored              */
} rcp_rot_kind;

/* Rotation descriptor (a host struct).  For RCP_ROT_KRON, x is viewed as an
 * n_wht x m row-major matrix X (k = i*m + j) and Y = H_{n_wht} X Q^T, which is
 * the standard Kronecker product H (x) Q applied to x.  Q is a DEVICE pointer to
 * an m x m row-major fp32 orthogonal matrix; it is ignored for the other kinds. */
typedef struct {
    int kind;       /* rcp_rot_kind                                                */
    int n_wht;      /* power of two: K for RCP_ROT_WHT, the Hadamard factor for KRON, the number of heads for HEADS */
    int m;          /* order of Q (1 for RCP_ROT_WHT); channels per head for HEADS   */
    const float* Q; /* device, m*m floats, row-major                               */
} rcp_rotation;

/* Limits of this build. */
#define RCP_MAX_M 16          /* tokens per call                                    */
#define RCP_MAX_ROTATE_ROWS 4096 /* rows per rcp_rotate_act call                      */
#define RCP_MAX_K 32768       /* input channels                                     */
#define RCP_MAX_WHT 16384     /* largest Hadamard order of a pure WHT rotation      */
#define RCP_MAX_KRON_M 256    /* largest order of Q                                 */
#define RCP_GROUP 128         /* input channels per unit of the group-wise calls    */

/* Library version, major*10000 + minor*100 + patch. */
int rcp_version(void);

/* Tuning knobs for benchmarks, sweeps and tests: a measurement hook outside the contract of the
 * compute calls, which keep no other state than the thread-local error string.  The knobs change how
 * work is spread over the GPU; integer results (packed bytes, x_q, S, partial sums) never depend on
 * them, binary32 / fp16 outputs only through "kv_tokens" (the split length of the attention sum fixes
 * its summation order, within the stated tolerance).  Value 0 restores the automatic choice of one
 * knob, rcp_set_option("reset", 0) that of all.  The settings are process-wide and are read by every
 * launch: do not change them while another host thread is inside a call.
 *   "gemv_lanes"   lanes that share one group of four rows: 16, 32, 64, 128, 256 (the kernel for group-wise tables
 *                  knows 32 = a lane owns whole quantisation groups, and 64 = two lanes share one, its automatic choice)
 *   "gemv_unroll"  16-byte loads per lane and pipeline stage: 2, 4
 *   "gemv_blocks"  number of workgroups the GEMV launches
 *   "gemv_variant" 1 = plain-ALU kernel for every M, 2 = matrix-core kernel for every M
 *   "gemm_waves"   wavefronts per workgroup of the matrix-core kernel: 1, 2, 4, 8
 *   "gemv_nt"      weight loads of the one-token kernels with the non-temporal cache hint (the one-shot form and the
 *                  forms with one wavefront or half a wavefront per group of rows): 1 = whenever such a form runs, 2 = never; automatic =
 *                  from 8 MB of packed weights on; the 3-bit kernel (from 16 MB on) and the kernel for
 *                  group-wise tables (from 4 MB on) and the weight-only kernel (from 4 MB on) likewise
 *   "gemm_stage"   128-column steps per pipeline stage of the matrix-core kernel: 1, 2 (automatic: 2 from eight steps
 *                  per wavefront on)
 *   "gemm_rows"    output rows per workgroup of the matrix-core kernel: 16 (four lanes per group of four rows), or
 *                  20, 24 .. 64 (one lane per group); automatic = 16 up to 8192 rows, else the smallest count that
 *                  gives every compute unit the same number of workgroups
 *   "kv_tokens"    cached tokens per workgroup of rcp_kv4_attn_decode: 64, 128, 256 (all loads of a workgroup
 *                  issued at once), 512, 1024, 2048 (the streaming kernel for long contexts and batches)
 *   "gemv_waves"   wavefronts per workgroup of the fused one-token GEMV (rcp_quant_w2a4_gemv): 4, 8
 *                  (8 needs K >= 2048 and "gemv_lanes" left automatic; otherwise 4 is used)
 *   "gemv_oneshot" one-token kernel that issues every weight load of a workgroup up front (one group of four rows
 *                  per wavefront, K <= 16384): 1 = for every such shape, 2 = never; automatic = matrices that give
 *                  every compute unit one or two workgroups, and with activations quantised beforehand every matrix
 *                  of at least one workgroup per unit with K >= 4096 below 32 MB.  Ignored while "gemv_lanes", "gemv_blocks" or
 *                  "gemv_unroll" is set (those address the general kernel).
 *   "seq_blocks"   workgroups of rcp_quant_w2a4_gemv_sequence (refused when they could not all be resident)
 *   "reset"        (value ignored) every knob back to automatic
 * Returns RCP_ERR_UNSUPPORTED for an unknown name or a value outside its set. */
int rcp_set_option(const char* name, int value);

/* Message for the last error on the calling thread (host string, never NULL). */
const char* rcp_last_error(void);

/* N*K/4, the size of the packed index buffer; 0 if the shape is not supported
 * (N must be a positive multiple of 4, K a positive multiple of 32). */
size_t rcp_packed_bytes(int N, int K);

/* Bytes of device scratch rcp_rotate_quant_act needs for this call shape
 * (0 when none is needed).  `rot` is a host pointer and may be NULL (= NONE). */
size_t rcp_act_workspace_bytes(int M, int K, const rcp_rotation* rot);

/*
 * Offline export (Section 4.3 "Partition"; LUT equation of Section 4.4).
 *
 * Per output row h with clip range [lo, hi] = [clip_lo[h], clip_hi[h]] (the
 * learned sigma(beta)*min and sigma(gamma)*max) and partition fractions
 * (p1, p2, p3) = part[3h .. 3h+2] (the learned sigma(s1), (1-p1)sigma(s2),
 * (1-p1)(1-sigma(s2)); they arrive as fractions so that no transcendental
 * function sits on the bit-exact path):
 *     range   = hi - lo
 *     t1 = p1/2,  t2 = t1 + (p1+p2)/2,  t3 = t2 + (p2+p3)/2      (grid t_i)
 *     w1 = (t1+t2)/2,  w2 = (t2+t3)/2                            (grid w_i)
 *     T_i = lo + range*t_i, rounded once to fp32
 *     idx[h][k] = [W >= T_1] + [W >= T_2] + [W >= T_3]           (Q_LDP, u(0)=1)
 *     LUT[h] = fp16( lo, lo + range*w1, lo + range*w2, hi )
 * All of the above is evaluated in IEEE double in the written order without
 * fused multiply-add, then rounded once (to nearest even).
 *
 * W: row-major N x K in `w_dtype`.  clip_lo, clip_hi: fp32 [N], lo < hi.
 * part: fp32 [N][3], each > 0.  packed_out: rcp_packed_bytes(N, K) bytes.
 * codebook_out: fp16 [N][4].  Values are not range-checked on the device.
 */
int rcp_pack_weights(const void* W, rcp_dtype w_dtype, int N, int K,
                     const float* clip_lo, const float* clip_hi, const float* part,
                     void* packed_out, void* codebook_out, void* stream);

/*
 * Online activation preparation.
 *     y      = R x                      (fp32 arithmetic; R from `rot`)
 *     a      = max_k |y_k|
 *     S      = fp16( clip_ratio * a / 7 ),  S = 1 when a == 0
 *     q_k    = clamp( round_half_even( y_k / S ), -8, 7 )
 * The Hadamard factor is the Sylvester matrix in natural order scaled by
 * 1/sqrt(n) (Appendix definition), with no random sign vector.
 * Activations must be finite: the codes of a token that holds an infinity or a NaN
 * are unspecified (here and in the calls that quantise in their prologue).
 *
 * x: row-major M x K in `x_dtype`.  rot: host pointer, NULL = RCP_ROT_NONE.
 * clip_ratio in (0, 1] (the paper's table uses 0.9).  xq_out: M*K/2 bytes.
 * scale_out: fp16 [M].  workspace: at least rcp_act_workspace_bytes(M, K, rot)
 * bytes of device scratch, may be NULL when that is 0.
 */
int rcp_rotate_quant_act(const void* x, rcp_dtype x_dtype, int M, int K,
                         const rcp_rotation* rot, float clip_ratio,
                         void* xq_out, void* scale_out,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * rcp_rotate_quant_act for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, arithmetic and results as rcp_rotate_quant_act (the same kernels run), but the scratch a
 * Kronecker rotation needs between its two kernels (M*K binary32 values) lives in a fixed array of
 * RCP_ACT_STATIC_SCRATCH_BYTES inside the library's device image -- each GPU the library runs on
 * holds that array until the process ends.  The call allocates nothing and frees nothing.
 * Returns RCP_ERR_WORKSPACE (nothing launched) when rcp_act_workspace_bytes(M, K, rot) exceeds
 * RCP_ACT_STATIC_SCRATCH_BYTES.  All calls on one GPU share the array: calls that may overlap on a GPU
 * (different streams, several host threads) race on it and must be serialised by the caller; calls on
 * one stream are ordered and safe.  Nothing in the array has to be cleared between calls (every value
 * read has been written by the same call).
 */
#define RCP_ACT_STATIC_SCRATCH_BYTES (1u << 20) /* 262144 binary32 values, e.g. 16 tokens x 14336 channels */
int rcp_rotate_quant_act_static(const void* x, rcp_dtype x_dtype, int M, int K,
                                const rcp_rotation* rot, float clip_ratio,
                                void* xq_out, void* scale_out, void* stream);

/*
 * The rotation step alone: y = R x in fp32 (the same kernels and arithmetic as the first half
 * of rcp_rotate_quant_act).  y_out: fp32 [M][K].  Meant to be followed by
 * rcp_quant_w2a4_gemv, which quantises in the prologue of the GEMV kernel.  M counts rows here and may
 * reach RCP_MAX_ROTATE_ROWS (e.g. the H_q query head vectors of a token, rotated one by one with K = 128).
 */
int rcp_rotate_act(const void* x, rcp_dtype x_dtype, int M, int K,
                   const rcp_rotation* rot, float* y_out, void* stream);

/*
 * Non-uniform W2A4 GEMV (M = 1) / skinny GEMM (M <= RCP_MAX_M), Section 4.4.
 *     P[m][h][l] = sum_{k : idx[h][k] = l} q[m][k]                (int32, exact)
 *     O[m][h]    = S[m] * sum_l LUT[h][l] * P[m][h][l]            (fp32)
 * which equals the paper's sum_k LUT[h][W_q[h][k]] * (S * X_q[k]).
 *
 * packed, codebook: as written by rcp_pack_weights.  xq, scale: as written by
 * rcp_rotate_quant_act.  out: M x N of `out_dtype` (RCP_F16 or RCP_F32).
 * partial_sums_or_null: when non-NULL receives int32 [M][N][4].
 * One token always runs on the vector ALUs (packed-int4 dot products on the bit planes), two
 * tokens too when N < 8192; two tokens with N >= 8192 and three or more tokens form the plane
 * sums on the matrix cores (the masked plane words are FP4 operands).  The per-level sums are
 * exact integers either way.  rcp_w2a4_gemv_variant reports that choice.
 */
int rcp_w2a4_gemv(const void* packed, const void* codebook, int N, int K,
                  const void* xq, const void* scale, int M,
                  void* out, rcp_dtype out_dtype,
                  int32_t* partial_sums_or_null, void* stream);

/* Which kernel rcp_w2a4_gemv runs for this shape under the current options (host only, nothing is
 * launched): 1 = vector-ALU kernel, 2 = matrix-core kernel; RCP_ERR_SHAPE for an unsupported shape. */
int rcp_w2a4_gemv_variant(int N, int K, int M);

/*
 * One-token fusion of the two calls above for an input that needs no online rotation
 * (or that is already rotated): the result is bit-identical to
 *     rcp_rotate_quant_act(x, 1 token, RCP_ROT_NONE, clip_ratio) -> rcp_w2a4_gemv(M = 1)
 * but the quantiser runs in the prologue of the GEMV kernel, so one launch is saved.
 * x: K values of `x_dtype`.  xq_out_or_null (K/2 bytes) and scale_out_or_null (one fp16)
 * receive the quantised activation the kernel used; both may be NULL for K <= 16384, for
 * larger K they are required (the call then runs the two kernels through them).
 */
int rcp_quant_w2a4_gemv(const void* packed, const void* codebook, int N, int K,
                        const void* x, rcp_dtype x_dtype, float clip_ratio,
                        void* out, rcp_dtype out_dtype,
                        void* xq_out_or_null, void* scale_out_or_null,
                        int32_t* partial_sums_or_null, void* stream);

/*
 * rcp_quant_w2a4_gemv with an online rotation inside the same launch: rot = NULL / RCP_ROT_NONE is
 * rcp_quant_w2a4_gemv; RCP_ROT_HEADS (K <= 16384) applies the Hadamard matrix across heads in
 * the prologue of the GEMV kernel and is bit-identical to rcp_rotate_quant_act(RCP_ROT_HEADS)
 * followed by rcp_w2a4_gemv; RCP_ROT_WHT with K <= 2048 (the order-K Hadamard rotation of a short input,
 * Appendix definition of H_n) runs in the prologue too, bit-identical to rcp_rotate_quant_act(RCP_ROT_WHT)
 * followed by rcp_w2a4_gemv.  Longer pure rotations and RCP_ROT_KRON return RCP_ERR_UNSUPPORTED: a long
 * transform over all of K would be repeated by every workgroup; run rcp_rotate_act first.  rot: host pointer.
 */
int rcp_rotate_quant_w2a4_gemv(const void* packed, const void* codebook, int N, int K,
                               const void* x, rcp_dtype x_dtype, const rcp_rotation* rot, float clip_ratio,
                               void* out, rcp_dtype out_dtype,
                               void* xq_out_or_null, void* scale_out_or_null,
                               int32_t* partial_sums_or_null, void* stream);

/*
 * Several dependent one-token GEMVs in ONE launch (Section 4.4; the layers of a decoder are applied one
 * after the other, Section 2.1 names the online rotation R_4 in front of the down projection).
 * Entry i computes exactly
 *     y_i   = rcp_rotate_act(x_i, rot_i)                    (rot_i: RCP_ROT_NONE or RCP_ROT_KRON)
 *     out_i = rcp_quant_w2a4_gemv(packed_i, codebook_i, N_i, K_i, y_i, clip_ratio_i)
 * bit for bit, in the order of the array, and entry i may read anything an earlier entry wrote (x_i may
 * point into out_j, j < i): all workgroups meet between consecutive entries, while the weights of the
 * next entry are already being fetched.  A caller that applies other operations between two linear
 * layers (attention, normalisation, gating) ends the sequence there.
 *
 * steps: HOST array of n entries, 1 <= n <= RCP_SEQ_MAX_STEPS, read before the call returns.  Per entry:
 * packed / codebook as written by rcp_pack_weights for N x K; x: K values of x_dtype (device);
 * rot.kind RCP_ROT_NONE, or RCP_ROT_KRON with n_wht in 64..1024 and (n_wht/64)*ceil(m/16) <= 16 (other
 * rotations: RCP_ERR_UNSUPPORTED); K <= 16384; out: N values of out_dtype (RCP_F16 / RCP_F32);
 * xq_out_or_null (K/2 bytes) / scale_out_or_null (one fp16) receive the quantised activation.
 * Buffers are 16-byte aligned; an output must not overlap any weight buffer or another output.
 *
 * workspace: rcp_gemv_sequence_workspace_bytes(steps, n) bytes of device memory that were ZERO when the
 * workspace was first used and have since been touched by this call only (the call leaves its
 * counters at zero again).  Word 0 (uint32) is an error flag: it stays 0 unless a wait inside the
 * kernel ran out of its bound -- only possible when the launch's workgroups were not all resident
 * at once, e.g. next to another kernel on the same GPU -- in which case the outputs are undefined and the
 * workspace has to be zeroed again.  Calls sharing a workspace must not overlap; sequences of different
 * length may share one (its layout does not depend on n), sized for the largest rotated K among them.  The grid (two
 * workgroups per compute unit, or "seq_blocks") is checked against the kernel's occupancy on the
 * host and refused with RCP_ERR_UNSUPPORTED when it could not be resident at once.
 */
#define RCP_SEQ_MAX_STEPS 16
typedef struct {
    const void* packed;      /* device */
    const void* codebook;    /* device, fp16 [N][4] */
    int N, K;
    const void* x;           /* device, K values of x_dtype */
    int x_dtype;             /* rcp_dtype */
    rcp_rotation rot;        /* RCP_ROT_NONE or RCP_ROT_KRON */
    float clip_ratio;        /* in (0, 1] */
    void* out;               /* device, N values of out_dtype */
    int out_dtype;           /* RCP_F16 or RCP_F32 */
    void* xq_out_or_null;    /* device, K/2 bytes */
    void* scale_out_or_null; /* device, one fp16 */
} rcp_gemv_step;
size_t rcp_gemv_sequence_workspace_bytes(const rcp_gemv_step* steps, int n);
int rcp_quant_w2a4_gemv_sequence(const rcp_gemv_step* steps, int n, void* workspace, size_t workspace_bytes,
                                 void* stream);

/*
 * Weight-only GEMV (the W2-only decode variant of the paper's inference-latency section:
 * non-uniform dequantisation merged into a 16-bit linear layer), one token:
 *     O[h] = sum_k LUT[h][idx[h][k]] * x[k]          (binary32 accumulation)
 * packed, codebook: as written by rcp_pack_weights.  x: K values of `x_dtype` (fp16 uses the
 * packed-fp16 dot instruction, bf16 / fp32 are widened to binary32).  out: N values of
 * `out_dtype` (RCP_F16 or RCP_F32).  K is limited by the activations having to fit in LDS:
 * K <= RCP_MAX_K for fp16, about 40000 values for the widened types (RCP_ERR_UNSUPPORTED).
 */
int rcp_w2a16_gemv(const void* packed, const void* codebook, int N, int K,
                   const void* x, rcp_dtype x_dtype,
                   void* out, rcp_dtype out_dtype, void* stream);

/* Measurement helper: read `bytes` (rounded down to 16) of a device buffer once with plain
 * 128-bit loads and discard them.  Timing it on a buffer of a GEMV's size gives the
 * streaming-read ceiling of the machine for a kernel of that size.  sink_or_null: 4 bytes of
 * device memory that are practically never written. */
int rcp_stream_read(const void* buffer, size_t bytes, void* sink_or_null, void* stream);

/* Verification helper: expand the packed indices to one byte per weight,
 * idx_out[h*K + k] in 0..3 (device, N*K bytes). */
int rcp_unpack_indices(const void* packed, int N, int K, uint8_t* idx_out, void* stream);

/*
 * Group-wise variants (Appendix table "Quantization configurations": weights quantised in
 * groups of 128 input channels; Section 4.4: LUT of N*4 entries per row for N groups).
 * `group` must be RCP_GROUP (RCP_ERR_UNSUPPORTED otherwise) and K a multiple of it.
 *
 * rcp_pack_weights_grouped: the export of rcp_pack_weights with one LDP grid per
 * (row, group).  clip_lo, clip_hi: fp32 [N][NG]; part: fp32 [N][NG][3]; packed_out: N*K/4
 * bytes in the grouped packed layout; codebook_out: N*NG*8 bytes in the grouped LUT layout.
 *
 * rcp_unpack_indices_grouped: grouped packed layout -> idx_out[h*K + k] in 0..3.
 *
 * rcp_w2a4_gemv_grouped (one token):
 *     P[h][g][l] = sum_{k in group g : idx[h][k] = l} q[k]              (int32, exact)
 *     O[h]       = S * sum_g sum_l LUT[h][g][l] * P[h][g][l]            (fp32 accumulation)
 * xq, scale: one token as written by rcp_rotate_quant_act.  out: N values of `out_dtype`.
 * partial_sums_or_null: when non-NULL receives int32 [N][NG][4].
 */
int rcp_pack_weights_grouped(const void* W, rcp_dtype w_dtype, int N, int K, int group,
                             const float* clip_lo, const float* clip_hi, const float* part,
                             void* packed_out, void* codebook_out, void* stream);
int rcp_unpack_indices_grouped(const void* packed, int N, int K, int group,
                               uint8_t* idx_out, void* stream);
int rcp_w2a4_gemv_grouped(const void* packed, const void* codebook, int N, int K, int group,
                          const void* xq, const void* scale,
                          void* out, rcp_dtype out_dtype,
                          int32_t* partial_sums_or_null, void* stream);
/* rcp_w2a4_gemm_grouped: the same product for M <= RCP_MAX_M tokens (xq: M x K/2 bytes, scale: fp16 [M],
 * out: M x N); several tokens run on the matrix cores, one step of the matrix instruction per
 * quantisation group.  partial_sums_or_null: int32 [M][N][NG][4]. */
int rcp_w2a4_gemm_grouped(const void* packed, const void* codebook, int N, int K, int group,
                          const void* xq, const void* scale, int M,
                          void* out, rcp_dtype out_dtype,
                          int32_t* partial_sums_or_null, void* stream);
/* rcp_quant_w2a4_gemv_grouped: the one-token fusion of rcp_quant_w2a4_gemv for group-wise LUTs,
 * bit-identical to rcp_rotate_quant_act (no rotation) followed by rcp_w2a4_gemv_grouped.
 * xq_out_or_null / scale_out_or_null as there (optional for K <= 16384, required beyond). */
int rcp_quant_w2a4_gemv_grouped(const void* packed, const void* codebook, int N, int K, int group,
                                const void* x, rcp_dtype x_dtype, float clip_ratio,
                                void* out, rcp_dtype out_dtype,
                                void* xq_out_or_null, void* scale_out_or_null,
                                int32_t* partial_sums_or_null, void* stream);

/*
 * 3-bit variant: LDP applied to the asymmetric normal-float 3-bit format (Section 4.3,
 * paragraph "Application of LDP on NF3 format": the centre point, the two scales of its
 * scale equation, the side-wise rounding of its quantisation equation, and dequantisation
 * as scale * grid value + centre).  The paper takes the format's grid from the work it
 * cites and does not print it; here the grid is an argument.
 *
 * rcp_pack_weights_w3: per output row h, in double precision,
 *     c = lo + (hi - lo) * frac,  s_neg = |c - lo|,  s_pos = |hi - c|
 *     L_j = c + (grid[j] < 0 ? s_neg : s_pos) * grid[j]     -> fp16, the LUT
 *     T_j = (L_{j-1} + L_j) / 2, j = 1..7                    -> fp32
 *     idx[h][k] = number of T_j <= W[h][k]                   (compared in fp32)
 *   which, when the grid holds 0, rounds (w - c)/s to the nearest grid value on w's side.
 *   W: N x K of `w_dtype`.  clip_lo, clip_hi, frac: fp32 [N] (the learnt clip values and the
 *   logistic of the learnt centre parameter).  grid: HOST pointer to eight strictly
 *   ascending finite floats (RCP_ERR_UNSUPPORTED otherwise).  packed_out: 3*N*K/8 bytes,
 *   codebook_out: N*16 bytes, in the 3-bit layouts above.
 * rcp_unpack_indices_w3: 3-bit packed layout -> idx_out[h*K + k] in 0..7 (N*K bytes).
 * rcp_w3a4_gemv (one token; the GEMV of Section 4.4 with an eight-entry LUT):
 *     P[h][l] = sum_{k : idx[h][k] = l} q[k]                 (int32, exact)
 *     O[h]    = S * sum_l LUT[h][l] * P[h][l]                (fp32, l ascending)
 *   xq, scale: one token as written by rcp_rotate_quant_act.  out: N values of `out_dtype`
 *   (RCP_F16 or RCP_F32).  partial_sums_or_null: when non-NULL receives int32 [N][8].
 *   The packed matrix must stay below 2 GiB (RCP_ERR_SHAPE).
 */
int rcp_pack_weights_w3(const void* W, rcp_dtype w_dtype, int N, int K,
                        const float* clip_lo, const float* clip_hi, const float* frac,
                        const float* grid_host,
                        void* packed_out, void* codebook_out, void* stream);
int rcp_unpack_indices_w3(const void* packed, int N, int K, uint8_t* idx_out, void* stream);
int rcp_w3a4_gemv(const void* packed, const void* codebook, int N, int K,
                  const void* xq, const void* scale,
                  void* out, rcp_dtype out_dtype,
                  int32_t* partial_sums_or_null, void* stream);
/* rcp_quant_w3a4_gemv: the per-token int4 quantiser of rcp_rotate_quant_act (no rotation; Appendix table of
 * quantisation configurations) fused into the prologue of rcp_w3a4_gemv: one launch instead of two, results
 * bit-identical to the two calls.  x: one token of K values of `x_dtype` (for a rotated input, the fp32 output
 * of rcp_rotate_act).  clip_ratio in (0, 1] (RCP_ERR_UNSUPPORTED otherwise).  xq_out_or_null (K/2 bytes) and
 * scale_out_or_null (fp16 [1]) receive x_q and S when given.  Other arguments as for rcp_w3a4_gemv. */
int rcp_quant_w3a4_gemv(const void* packed, const void* codebook, int N, int K,
                        const void* x, rcp_dtype x_dtype, float clip_ratio,
                        void* out, rcp_dtype out_dtype,
                        void* xq_out_or_null, void* scale_out_or_null,
                        int32_t* partial_sums_or_null, void* stream);

/* ---------------------------------------------------------------------------------------
 * 4-bit KV cache and one-token attention over it.  Appendix, table of quantisation
 * configurations: the KV cache uses an asymmetric quantiser on groups of 128 with clipping
 * ratio 0.95; the quantiser is Eqn. 1 with N = 4.  Section 2.1: the online rotation R3 is
 * applied to queries and keys so that the cache can be held in 4 bits without changing the
 * attention output: rcp_kv4_append applies it to the keys when `rotate` is set, and the query
 * goes through rcp_rotate_act (an order-128 WHT over H_q rows of 128) before rcp_kv4_attn_decode.
 * Head size is RCP_KV_HEAD_DIM = 128 = one group.
 *
 * Layout of one cached tensor (keys or values) of one layer, both device buffers, caller-owned:
 *   codes   [H][S_max][64 bytes]  element j of a head vector in byte j / 2, bits 4*(j%2) .. 4*(j%2)+3
 *   params  [H][S_max][4 bytes]   bytes 0..1 the binary16 step size s, bytes 2..3 the int16 zero point z
 * A code c stands for the value s * (c - z).
 *
 * rcp_kv4_append: x is [n_tokens][H][128] of `x_dtype`; token i goes to cache position pos + i
 *   (0 <= pos, pos + n_tokens <= S_max, else RCP_ERR_SHAPE; n_tokens = 0 is a no-op).  rotate != 0: every head
 *   vector is first replaced by its normalised order-128 Hadamard transform, computed in binary32 with the
 *   butterflies in ascending stride order and one multiplication by (float)(1/sqrt(128)) (keys; values are
 *   stored unrotated here, their rotation being folded into the projection weights).  Then, in binary32:
 *     lo = ratio * min(x), hi = ratio * max(x), s = fp16((hi - lo) / 15)   [1 when that is 0; capped at 65504]
 *     z = -rint(lo / s)  [clamped to int16],  c_j = clamp(rint(x_j / s) + z, 0, 15)
 *   with correctly rounded divisions and round-half-to-even.  Other cache positions are not touched.
 *   The one clipping ratio scales the minimum and the maximum (the form of the paper's clipping equation):
 *   the range of a group whose values all have one sign moves towards zero instead of shrinking about the
 *   data, and what lies beyond ratio*max (ratio*min) takes the end code -- harmless for rotated keys and
 *   values, which are centred near zero; pass clip_ratio = 1 for data that is not.  z is held in 16 bits: a group
 *   with |lo / s| above 32767 (a range 2000 times narrower than its offset) saturates z and is misrepresented.
 *   pos, n_tokens (and S below) are call arguments that the kernels receive by value: a captured HIP graph
 *   replays the positions and lengths it was captured with, so a decode loop under graph capture must update
 *   these kernel-node arguments (or re-capture) every step.
 * rcp_kv4_attn_decode: one query token against cache positions 0 .. S-1 (1 <= S <= S_max):
 *     out[h] = sum_t softmax_t(softmax_scale * q[h] . K[g][t]) * V[g][t],   g = h / (H_q / H_kv)
 *   q: [H_q][128] of `q_dtype`; out: [H_q][128] of `out_dtype` (RCP_F16 or RCP_F32); H_q a multiple of
 *   H_kv.  Sums are binary32.  workspace: rcp_kv4_workspace_bytes(H_q, S) bytes of device memory
 *   (RCP_ERR_WORKSPACE when missing or smaller; the size covers every "kv_tokens" setting), overwritten by every call.  S above
 *   RCP_KV_MAX_S returns RCP_ERR_UNSUPPORTED.
 */
#define RCP_KV_HEAD_DIM 128
#define RCP_KV_MAX_S 262144
size_t rcp_kv4_workspace_bytes(int H_q, int S);
int rcp_kv4_append(const void* x, rcp_dtype x_dtype, int n_tokens, int H, int S_max, int pos,
                   int rotate, float clip_ratio, void* codes, void* params, void* stream);
int rcp_kv4_attn_decode(const void* q, rcp_dtype q_dtype, int H_q, int H_kv, int S_max, int S,
                        const void* k_codes, const void* k_params,
                        const void* v_codes, const void* v_params,
                        float softmax_scale, void* out, rcp_dtype out_dtype,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Fewer launches for a decode step over the 4-bit cache (same arithmetic, same bits as the calls above):
 * rcp_kv4_append_kv: the new keys and the new values of the same n_tokens tokens in ONE launch -- exactly
 *   rcp_kv4_append(k, ..., rotate_k, clip_ratio, k_codes, k_params) and rcp_kv4_append(v, ..., 0, clip_ratio, v_codes, v_params).
 *   k and v: [n_tokens][H][128] of `x_dtype`.
 * rcp_kv4_rotate_attn_decode: rcp_kv4_attn_decode on the UN-rotated query: the order-128 Hadamard rotation R3 of every
 *   query head runs inside the attention kernel (while the cache loads are in flight), bit for bit what rcp_rotate_act
 *   (RCP_ROT_WHT, n = 128, over the H_q rows of q) followed by rcp_kv4_attn_decode on its binary32 output gives.
 */
int rcp_kv4_append_kv(const void* k, const void* v, rcp_dtype x_dtype, int n_tokens, int H, int S_max, int pos,
                      int rotate_k, float clip_ratio, void* k_codes, void* k_params, void* v_codes, void* v_params,
                      void* stream);
int rcp_kv4_rotate_attn_decode(const void* q, rcp_dtype q_dtype, int H_q, int H_kv, int S_max, int S,
                               const void* k_codes, const void* k_params, const void* v_codes, const void* v_params,
                               float softmax_scale, void* out, rcp_dtype out_dtype,
                               void* workspace, size_t workspace_bytes, void* stream);

/* Several sequences at once (the small-batch decode of Section 4.4's GEMM discussion applied to the cache):
 * B <= RCP_MAX_M sequences share pooled buffers, sequence b owning heads b*H .. b*H + H - 1 of
 * codes [B*H][S_max][64] / params [B*H][S_max][4].  pos_host / S_host are HOST arrays of B ints, read
 * before the call returns.
 * rcp_kv4_append_batched: x is [B][H][128]; row b is the new token of sequence b and goes to its position
 *   pos_host[b] (0 <= pos_host[b] < S_max, else RCP_ERR_SHAPE).  Arithmetic as rcp_kv4_append.
 * rcp_kv4_attn_decode_batched: q and out are [B][H_q][128]; sequence b attends to its first S_host[b] tokens
 *   (1 <= S_host[b] <= S_max).  Each row equals what rcp_kv4_attn_decode gives for that sequence alone
 *   up to the order of its binary32 sums: the automatic split length is chosen from the total number of
 *   cached tokens of the call, so a batched row and the single call agree bit for bit only when the
 *   "kv_tokens" option fixes the split length, and within the stated tolerance otherwise.  workspace: B * rcp_kv4_workspace_bytes(H_q, max_b S_host[b])
 *   bytes.  H_q <= 4095. */
int rcp_kv4_append_batched(const void* x, rcp_dtype x_dtype, int B, int H, int S_max, const int* pos_host,
                           int rotate, float clip_ratio, void* codes, void* params, void* stream);
int rcp_kv4_attn_decode_batched(const void* q, rcp_dtype q_dtype, int B, int H_q, int H_kv, int S_max,
                                const int* S_host,
                                const void* k_codes, const void* k_params,
                                const void* v_codes, const void* v_params,
                                float softmax_scale, void* out, rcp_dtype out_dtype,
                                void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RCP_H */
