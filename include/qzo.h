/*
 * qzo.h -- C ABI of the MI355X (gfx950) hot path of Quantized Zeroth-order
 * Optimization (QZO): two perturbed forward passes through a weight-quantized
 * decoder, the SPSA directional derivative, its clipping, and the in-place
 * update of the quantization scales (paper Sec. 3.2: Def. 3.3 / Eq. 5
 * "Q-SPSA", Eq. 6 "DDC", Algorithm 1).
 *
 * Conventions
 *  - Every pointer named *_dev is DEVICE memory owned by the caller; the
 *    library borrows it for the duration of the call (model tensors and the
 *    scale arena: for the lifetime of the model).  Pointers not so named are
 *    host memory.  Device pointers must be 16-byte aligned.
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and returns without synchronising.  Results stay on
 *    the device.
 *  - Every function returns QZO_OK or a negative qzo_status and qzo_last_error()
 *    describes the reason (thread-local string, valid until the next failing call
 *    on that thread).  Arguments, shapes, alignment, workspace and scratch sizes and
 *    the kernels' 32-bit addressing limits are all checked before the first launch:
 *    a call that fails with any status other than QZO_ERR_HIP has enqueued nothing.
 *    QZO_ERR_HIP reports a failing HIP runtime call (a launch the runtime refused);
 *    launches issued before it stay enqueued.
 *  - The library allocates no device memory: every buffer, including scratch, is the
 *    caller's.  The measurement hooks create HIP events.
 *  - bf16 = upper 16 bits of an IEEE fp32, round-to-nearest-even on store.
 *
 * Data layout
 *  - Quantized weight of a linear with N outputs and K inputs: packed int4,
 *    uint8 [N, K/2], K contiguous; byte j of row n holds column 2j in its low
 *    nibble and 2j+1 in its high nibble; stored nibble = integer weight + 8
 *    (integer weight in [-8, 7], the paper's w-bar of Eq. 3).
 *  - Its scales (the paper's Delta): bf16 [N, K/group], group = 128 consecutive
 *    input features of one output row; dequantization is Eq. 4, w = Delta*w-bar.
 *  - Perturbation noise z is never stored.  z for (row r, group g) is a pure
 *    function of (seed, r, g): Philox4x32-10 with key = seed and counter =
 *    (r, g/8, stream_id, 0); each 32-bit output word yields one Box-Muller
 *    pair, so one counter serves groups 8*(g/8) .. 8*(g/8)+7 of row r.  r is
 *    the row's index in the model-wide enumeration of quantized output rows
 *    (`row_base` of a tensor + row within the tensor).
 */
#ifndef QZO_H_
#define QZO_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  QZO_OK = 0,
  QZO_ERR_ARG = -1,        /* null pointer, bad enum, negative clip, sign not +-1 ... */
  QZO_ERR_SHAPE = -2,      /* dimension not supported by the kernels */
  QZO_ERR_ALIGN = -3,      /* device pointer not 16-byte aligned */
  QZO_ERR_WORKSPACE = -4,  /* workspace too small */
  QZO_ERR_NONFINITE = -5,  /* reported in qzo_step_result.status only */
  QZO_ERR_HIP = -6,        /* a HIP runtime call failed */
  QZO_ERR_UNSUPPORTED = -7
} qzo_status;

typedef struct qzo_model qzo_model; /* opaque, host object owned by the library */

typedef struct {
  uint32_t struct_size; /* sizeof(qzo_model_config), for versioning */
  uint32_t arch;        /* 0: Llama family (RMSNorm, RoPE, SwiGLU, no bias)
                           1: OPT family (LayerNorm, learned positions, ReLU, biases) */
  uint32_t n_layers, d_model, n_heads, d_ffn, vocab, max_seq;
  uint32_t group_size;  /* 128; 64 with quant = 3 */
  uint32_t quant;       /* 0: int4 + per-group bf16 scales
                           1: codebook (Llama only): one uint16 code per 8 weights into a per-linear
                              fp16 [65536,8] codebook, fp16 per-output-channel scales
                           2: int4 + per-group bf16 scales + per-group zero-points,
                              W = s * (u - zp) (Sec. 4.1, quantizers that keep a zero-point)
                           3: 4-bit NormalFloat indices + one bf16 scale per block of 64
                              (group_size = 64), W = s * level[u] (Sec. 4.3's quantizer) */
  float norm_eps;       /* 1e-5 */
  float rope_theta;     /* 10000 (Llama only) */
  uint32_t scale_fp16;  /* quant 0 and 2: 0 = the group scales of the arena are bf16, 1 = fp16 (the scale
                           type of the 4-bit checkpoints of Sec. 4.1; with the paper's eta = 1e-7 a bf16
                           arena rounds nearly every update away, an fp16 arena does not) */
  uint32_t act_order;   /* quant 2 only: 1 = every zero-point tensor of the table is followed by g_idx,
                           int32 [K], the group of each input column (activation reordering); such a
                           linear always runs expand-then-multiply */
} qzo_model_config;

typedef struct {
  const void* ptr_dev;
  uint64_t bytes;
} qzo_buf;

typedef struct {
  float loss_plus, loss_minus; /* l+ and l- of Algorithm 1 */
  float d;                     /* (l+ - l-) / (2 eps) */
  float d_clipped;             /* Eq. 6 */
  int32_t status;              /* QZO_OK, or QZO_ERR_NONFINITE: d not finite, update skipped */
  uint32_t reserved[3];
} qzo_step_result;

/*
 * Binds a model to caller-owned device tensors (Algorithm 1's inputs: scales
 * Delta, quantized weights theta-bar).  `tensors` lists, in forward order:
 *   Llama: tok_emb bf16[V,d]; per layer { attn_norm bf16[d], wqkv int4[3d,d/2],
 *          wo int4[d,d/2], ffn_norm bf16[d], wgu int4[2F,d/2] (gate rows, then up
 *          rows), wdown int4[d,F/2] }; final_norm bf16[d]; lm_head bf16[V,d].
 *   OPT:   tok_emb; pos_emb bf16[max_seq,d]; per layer { ln1_g, ln1_b bf16[d],
 *          wqkv int4[3d,d/2], bqkv bf16[3d], wo int4[d,d/2], bo bf16[d], ln2_g, ln2_b,
 *          wfc1 int4[F,d/2], bfc1 bf16[F], wfc2 int4[d,F/2], bfc2 bf16[d] };
 *          lnf_g, lnf_b; lm_head bf16[V,d].
 *   Llama, quant = 1: per layer { attn_norm, codes_qkv uint16[3d,d/8], cb_qkv fp16[65536,8],
 *          codes_o, cb_o, ffn_norm, codes_gu [2F,d/8], cb_gu, codes_down [d,F/8], cb_down };
 *          the arena then holds one fp16 scale per output row, per layer [3d][d][2F][d].
 *   quant = 2 (either family): the quant = 0 table with every int4 weight [N,K/2] directly
 *          followed by its zero-points uint8 [N,K/128], values 0..15, and with act_order = 1 by its
 *          group index int32 [K] (values 0 .. K/128 - 1; column k of the linear belongs to group
 *          g_idx[k] instead of k/128; scales, zero-points and noise stay per (row, group)); scales
 *          and the arena as for quant = 0.
 *   quant = 3 (either family): the quant = 0 table with NormalFloat-4 indices in place of the int4
 *          nibbles (same [N,K/2] layout, even k in the low nibble); the arena holds [N, K/64] scales
 *          per linear.  Every linear is first written out as a perturbed bf16 matrix in the workspace
 *          and multiplied by a plain bf16 GEMM.
 * `scale_arena_dev` holds every quantized linear's scales (bf16, or fp16 with
 * scale_fp16 = 1) back to back in the same order ([N, K/128] each); it is the only
 * model memory the library writes.  Only the decoder-block linears are quantized and trained (their
 * scale count is the paper's Table 2 "trainable parameters"); embeddings,
 * norms, biases and lm_head are fixed bf16.  Row ids for the noise follow the
 * arena order.  Requires d_model % 128 == 0, d_ffn % 128 == 0,
 * d_model/n_heads in {64, 128}.  Host work only: nothing is allocated or enqueued on
 * the device (the RoPE angle table lives in the workspace and is rebuilt by every pass).
 * QZO_ERR_SHAPE also when a linear of the model is too large for the kernels' 32-bit
 * byte offsets (N*K*2 bytes of one expanded linear must stay below 2^31).
 */
qzo_status qzo_model_create(const qzo_model_config* cfg, const qzo_buf* tensors,
                            uint32_t n_tensors, void* scale_arena_dev, uint64_t n_scales,
                            qzo_model** out);
qzo_status qzo_model_destroy(qzo_model* m);

/* Number of quantization scales a config has (host arithmetic only). */
qzo_status qzo_model_scale_count(const qzo_model_config* cfg, uint64_t* out);

/* Bytes of device workspace qzo_forward_loss / qzo_step need for (batch, seq): activations,
 * cross-entropy partials, the RoPE angle table, K-slice partial sums, and for the
 * expand-then-multiply route (see qzo_model_set_int4_path) one linear's perturbed weights in
 * bf16 plus every perturbed scale of the model in fp32.  Depends on the model's int4 route and
 * on joint mode: query it after setting those. */
qzo_status qzo_workspace_bytes(const qzo_model* m, uint32_t batch, uint32_t seq, uint64_t* out);

/*
 * One perturbed forward pass: L((Delta + sign*eps*z) (.) theta-bar; B) of Eq. 5,
 * next-token cross-entropy averaged over the batch*(seq-1) predicted positions.
 * The stored scales are not modified: the perturbed scale s + sign*eps*z is one fp32
 * fma (the functional form of PERTURB_SCALES in Algorithm 1), formed inside the GEMM's
 * weight tile on the fused route.  On the expand-then-multiply route (the default from a
 * few thousand tokens per pass on, see qzo_model_set_int4_path) a pass first writes the
 * perturbed scales of the whole model (fp32) and then, linear by linear, the perturbed
 * weights (bf16) into the workspace, where they live until the next linear / pass
 * overwrites them; z itself is never written anywhere.
 * tokens_dev: int32 [batch, seq], values in [0, vocab).
 * loss_dev: one fp32.  seq <= max_seq.  sign must be +1 or -1.
 */
qzo_status qzo_forward_loss(qzo_model* m, const int32_t* tokens_dev, uint32_t batch,
                            uint32_t seq, uint64_t seed, float eps, int sign,
                            void* workspace_dev, uint64_t workspace_bytes, float* loss_dev,
                            void* stream);

/*
 * One iteration of Algorithm 1: l+ and l- from two perturbed forwards with the
 * same seed, d = (l+ - l-)/(2 eps), d' = clip(d, -C, C) (Eq. 6), then
 * Delta_i <- max(Delta_i - eta*d'*z_i, 0) over the whole arena with z
 * regenerated from `seed`.  No host synchronisation inside; result_dev
 * receives the scalars.  clip must be >= 0.  A non-finite d leaves the scales
 * untouched and sets result.status = QZO_ERR_NONFINITE.
 * With int4 weights (no joint mode, no group index per column) the two forwards run as one
 * forward over 2*batch sequences when batch*seq <= 32 (the few-token kernel then reads the
 * weights once for both passes; losses bit-identical to two qzo_forward_loss calls) or when
 * batch*seq is above 64 and below the token count from which the model's linears take the
 * expand-then-multiply route (about 3200 at Llama-2-7B widths; at most 4096; never when that
 * route is forced): a launch of the tile kernel then holds the token tiles of both passes, the
 * second pass's with -eps and starting on a 256-row tile boundary (padding rows in between);
 * losses equal to two qzo_forward_loss calls within the 16-bit activations' noise, the K split
 * of a linear being a function of the number of token tiles.  qzo_workspace_bytes accounts for it.
 */
qzo_status qzo_step(qzo_model* m, const int32_t* tokens_dev, uint32_t batch, uint32_t seq,
                    uint64_t seed, float eps, float eta, float clip, void* workspace_dev,
                    uint64_t workspace_bytes, qzo_step_result* result_dev, void* stream);

/*
 * Joint mode (Sec. 3.2: Q-SPSA on the scales combined with SPSA, Def. 3.1, on the parameters that
 * were never quantized; the 2-bit runs of Sec. 4.1 train both).  The un-quantized parameters
 * theta_u are every 16-bit tensor of the model table (embeddings, norm gains and biases, lm_head;
 * with quant = 1 also the fp16 codebooks), concatenated in table order into one caller-owned
 * fp32 master vector dense_master_dev [n_dense], n_dense = qzo_model_dense_count(cfg).  Entry i
 * draws z_i from the step's seed on a stream of its own (stream 2, Philox counter (i/8, 0)).
 *
 * After qzo_model_enable_joint the table's 16-bit tensors are derived data that the library
 * WRITES: every forward first sets each of them to round16(theta_u + sign*eps*z) (one fp32 fma, one
 * round-to-nearest-even to the tensor's bf16 or fp16), and qzo_step_joint ends by
 *   theta_u <- theta_u - eta_dense * d' * z   (fp32, one fma, no clamp at zero)
 * next to the scale update, and by bringing the 16-bit tensors back to round16(theta_u).  The
 * master and the tensors must stay valid and unaliased for the model's lifetime; the caller
 * initialises the master (normally from the 16-bit tensors).  The two perturbed passes are never
 * stacked in joint mode.  table_dev: qzo_model_joint_table_bytes(cfg) bytes of caller-owned device
 * memory (16-byte aligned) that receives one entry per 16-bit tensor and must stay valid and
 * untouched for the model's lifetime; qzo_model_enable_joint fills it with a synchronous
 * host-to-device copy (a set-up call: the only one in this library that synchronises).
 * Errors: QZO_ERR_SHAPE if n_dense is not the config's count, QZO_ERR_ALIGN if the master or the
 * table is not 16-byte aligned, QZO_ERR_WORKSPACE if the table is too small, QZO_ERR_ARG if joint
 * mode is already on; qzo_step refuses a model in joint mode and qzo_step_joint one that is not.
 */
qzo_status qzo_model_dense_count(const qzo_model_config* cfg, uint64_t* out);
qzo_status qzo_model_joint_table_bytes(const qzo_model_config* cfg, uint64_t* out);
qzo_status qzo_model_enable_joint(qzo_model* m, float* dense_master_dev, uint64_t n_dense,
                                  void* table_dev, uint64_t table_bytes);
qzo_status qzo_step_joint(qzo_model* m, const int32_t* tokens_dev, uint32_t batch, uint32_t seq,
                          uint64_t seed, float eps, float eta, float eta_dense, float clip,
                          void* workspace_dev, uint64_t workspace_bytes,
                          qzo_step_result* result_dev, void* stream);

/* The update loop of Algorithm 1 alone over the model's arena, with d' given by
 * the host (eta*d' formed as one fp32 product). */
qzo_status qzo_model_apply_update(qzo_model* m, uint64_t seed, float eta, float d_clipped,
                                  void* stream);

/*
 * A single perturbed W4A16 linear (Eq. 4-5): Y = X * W_eff^T with
 * W_eff[n,k] = (s[n,k/group] + sign*eps*z(row_base+n, k/group)) * wbar[n,k].
 * x_dev bf16 [M,K] row-major; q_dev packed int4 [N,K/2]; s_dev bf16 [N,K/group];
 * y_dev bf16 [M,N].  sumsq_dev (nullable): one fp32 receiving sum_{m,n} y^2 of
 * the bf16-rounded outputs.  Requires group == 128, K % 128 == 0, N % 8 == 0.
 * scratch_dev: qzo_linear_scratch_bytes(M, N, K, sumsq_dev != NULL) bytes of caller-owned
 * device memory, 256-byte aligned (may be NULL when that size is 0), contents undefined
 * afterwards; calls that share a scratch buffer must not overlap.  It holds the per-tile
 * partial sums of sum y^2 and the K-slice partial sums of the two paths below.
 * With M <= 64 the call takes the few-token path (the paper's batch-1 memory
 * profile and short-prompt batches, Sec. 4.3): the int4 weights are streamed once and
 * enter the matrix unit as integer codes, each 128-wide group's sum is scaled by the
 * perturbed scale in fp32 (Eq. 4-5 without a bf16 rounding of the weights),
 * K is split over workgroups (slices of 8 groups, 4 for small outputs) and the fp32
 * partial sums (slices * M * N floats) are added in slice order (deterministic).
 * Inside a model the same path uses the workspace.
 * With more tokens but fewer than half as many 256 x 256 output tiles as the chip has compute units,
 * the tile kernel also splits K (slices of a multiple of 256 input features, at most
 * compute units / tiles of them) and a second kernel adds the slices in slice order.
 * QZO_ERR_WORKSPACE if scratch_bytes is too small, QZO_ERR_SHAPE if an operand exceeds
 * the kernels' 32-bit byte offsets (M*K*2, N*K/2 or M*N*2 bytes >= 2^31).
 */
qzo_status qzo_linear_scratch_bytes(uint32_t M, uint32_t N, uint32_t K, int with_sumsq, uint64_t* out);
qzo_status qzo_dequant_gemm(const void* x_dev, const void* q_dev, const void* s_dev,
                            uint32_t row_base, uint32_t M, uint32_t N, uint32_t K,
                            uint32_t group, uint64_t seed, float eps, int sign, void* y_dev,
                            float* sumsq_dev, void* scratch_dev, uint64_t scratch_bytes,
                            void* stream);

/*
 * qzo_dequant_gemm for callers that cannot allocate device memory and have no scratch to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operands,
 * same kernels and bit-identical results; the scratch is a fixed 32 MiB array that is part of the
 * loaded library (every GPU the library is used on holds its own copy until the process ends), so
 * the call allocates nothing.  The calling thread's current device must be the one the pointers and
 * the stream belong to.  QZO_ERR_WORKSPACE when qzo_linear_scratch_bytes(M, N, K, sumsq_dev != NULL)
 * exceeds 32 MiB (at M <= 64 that is N up to about 16000 at 8 K slices, any of the Llama-2-7B / 13B
 * linears; the single-linear workload 2048 x 11008 x 4096 needs 1.5 KB); then nothing is enqueued.
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents: calls that
 * overlap on one GPU (two streams, two threads) race, and must be serialised by the caller.
 */
qzo_status qzo_dequant_gemm_static(const void* x_dev, const void* q_dev, const void* s_dev,
                                   uint32_t row_base, uint32_t M, uint32_t N, uint32_t K,
                                   uint32_t group, uint64_t seed, float eps, int sign, void* y_dev,
                                   float* sumsq_dev, void* stream);

/*
 * The same linear for asymmetric 4-bit groups, the format of the 4-bit checkpoints the paper
 * fine-tunes (Sec. 4.1: group-128 quantizer with zero-points):
 *   W_eff[n,k] = (s[n,k/group] + sign*eps*z(row_base+n, k/group)) * (u[n,k] - zp[n,k/group])
 * with the stored nibble u in 0..15 and zp_dev uint8 [N, K/group] holding integer zero-points
 * 0..15 (zp = 8 everywhere is qzo_dequant_gemm).  The integer difference is formed exactly and
 * multiplied once, so the bf16 weight tile equals the definition bit for bit.  Everything
 * else (layouts, sumsq_dev, the few-token path, scratch) as in qzo_dequant_gemm.  The trained
 * quantities are the scales; zero-points are fixed.  scale_fp16: 0 = s_dev holds bf16, 1 = fp16.
 */
qzo_status qzo_dequant_gemm_zp(const void* x_dev, const void* q_dev, const void* s_dev,
                               const void* zp_dev, uint32_t scale_fp16, uint32_t row_base, uint32_t M,
                               uint32_t N, uint32_t K, uint32_t group, uint64_t seed, float eps, int sign,
                               void* y_dev, float* sumsq_dev, void* scratch_dev,
                               uint64_t scratch_bytes, void* stream);

/*
 * Repacks an asymmetric 4-bit linear from the K-major layout such checkpoints are stored in:
 *   qweight_dev int32 [K/8, N]   word (kk, n) = nibbles of k = 8 kk .. 8 kk + 7 of output n, lowest first
 *   qzeros_dev  int32 [K/group, N/8]  word (g, nn) = zero-points of n = 8 nn .. 8 nn + 7, lowest first
 *   scales_dev  fp16  [K/group, N]
 * into this library's layout: q_dev bytes [N, K/2], zp_dev uint8 [N, K/group] = (stored zero-point
 * + zero_add) & 15 (some writers store the zero-point minus one: zero_add = 1), s_dev
 * [N, K/group] = the fp16 scale itself (scale_fp16 = 1) or rounded to nearest even to bf16 (0).
 * group == 128, K % 128 == 0, N % 8 == 0.  A checkpoint's group index (activation reordering) needs
 * no repacking: it is handed to the model table as it is.
 */
qzo_status qzo_repack_kmajor(const void* qweight_dev, const void* qzeros_dev, const void* scales_dev,
                             uint32_t N, uint32_t K, uint32_t group, uint32_t zero_add,
                             uint32_t scale_fp16, void* q_dev, void* zp_dev, void* s_dev, void* stream);

/*
 * Codebook variant of the perturbed linear (the paper's 2-bit setting, Sec. 3.2.1 last
 * paragraph / Sec. 4.1: 1 codebook of 16 bits, channel-wise scales trained by QZO):
 *   W[n,k] = c[n] * CB[codes[n,k/8]][k%8],  Y = (X * (CB-weights)^T) * diag(c + sign*eps*z)
 * with z(row_base + n) from the flat noise stream 1 (counter ((row_base+n)/8, 0, 1, 0)).
 * x_dev bf16 [M,K]; codes_dev uint16 [N,K/8]; codebook_dev fp16 [65536,8]; c_dev fp16 [N];
 * y_dev bf16 [M,N]; sumsq_dev as in qzo_dequant_gemm.  K % 128 == 0, N % 8 == 0.  Codebook
 * entries are rounded to bf16 for the MFMA; the scale multiplies the fp32 accumulators.
 * scratch_dev: qzo_codebook_scratch_bytes(M, N, sumsq_dev != NULL) bytes (256-byte aligned,
 * NULL allowed when 0): one float per output tile for sum y^2.
 */
qzo_status qzo_codebook_scratch_bytes(uint32_t M, uint32_t N, int with_sumsq, uint64_t* out);
qzo_status qzo_codebook_gemm(const void* x_dev, const void* codes_dev, const void* codebook_dev,
                             const void* c_dev, uint32_t row_base, uint32_t M, uint32_t N, uint32_t K,
                             uint64_t seed, float eps, int sign, void* y_dev, float* sumsq_dev,
                             void* scratch_dev, uint64_t scratch_bytes, void* stream);
/* c_n <- max(c_n - eta*d'*z_n, 0) on fp16 channel scales c_dev[n_rows], round-to-nearest-even. */
qzo_status qzo_apply_update_channel(void* c_dev, uint32_t n_rows, uint32_t row_base, uint64_t seed,
                                    float eta, float d_clipped, void* stream);

/* The update loop of Algorithm 1 on one tensor's scales: s_dev [n_rows, G], bf16 (scale_fp16 = 0) or
 * fp16 (1), updated in place with c = eta*d_clipped and rounded to nearest even in that type. */
qzo_status qzo_apply_update(void* s_dev, uint32_t n_rows, uint32_t G, uint32_t row_base,
                            uint64_t seed, float eta, float d_clipped, uint32_t scale_fp16, void* stream);

/* RTN quantizer of Eq. 3 with the k=4 absmax scale: w_dev fp32 [N,K] ->
 * q_dev packed int4 [N,K/2], s_dev bf16 [N,K/group].  Model construction, not
 * part of the timed step. */
qzo_status qzo_rtn_quantize(const float* w_dev, uint32_t N, uint32_t K, uint32_t group,
                            void* q_dev, void* s_dev, void* stream);
/* The same with a zero-point (Eq. 3 on the group's range, which always includes 0): the scale is
 * round16((max - min) / 15), the zero-point rne(-min / scale) clamped to 0..15, the nibble
 * clamp(rne(w / scale) + zero-point, 0, 15); an all-zero group gets scale 0, zero-point 8, nibbles 8.
 * q_dev packed nibbles [N,K/2], zp_dev uint8 [N,K/group], s_dev [N,K/group] in bf16 (scale_fp16 = 0)
 * or fp16 (1).  group == 128. */
qzo_status qzo_rtn_quantize_asym(const float* w_dev, uint32_t N, uint32_t K, uint32_t group,
                                 uint32_t scale_fp16, void* q_dev, void* zp_dev, void* s_dev, void* stream);

/* Inspection entry points used by the parity tests. */
/* out_dev fp32 [n_rows, G] = z(row0 + r, g), noise stream `stream_id` (0 = group scales). */
qzo_status qzo_debug_normals(uint64_t seed, uint32_t stream_id, uint32_t row0, uint32_t n_rows,
                             uint32_t G, float* out_dev, void* stream);
/* out_dev uint32 [n,4] = Philox4x32-10(ctr = ctr_dev[i][0..3], key = seed). */
qzo_status qzo_debug_philox(uint64_t seed, const uint32_t* ctr_dev, uint32_t n,
                            uint32_t* out_dev, void* stream);
/* out_dev fp32 [n,2] = the normal pair of each 32-bit word. */
qzo_status qzo_debug_normal_pairs(const uint32_t* words_dev, uint32_t n, float* out_dev,
                                  void* stream);
/* w_eff_dev bf16 [N,K] = bf16((s + sign*eps*z) * wbar), the GEMM's B operand. */
qzo_status qzo_debug_dequant(const void* q_dev, const void* s_dev, uint32_t row_base, uint32_t N,
                             uint32_t K, uint32_t group, uint64_t seed, float eps, int sign,
                             void* w_eff_dev, void* stream);
/* The same with zero-points (zp_dev uint8 [N, K/group], nullable = 8) and bf16 or fp16 scales: the B
 * operand of qzo_dequant_gemm_zp. */
qzo_status qzo_debug_dequant_zp(const void* q_dev, const void* s_dev, const void* zp_dev,
                                uint32_t scale_fp16, uint32_t row_base, uint32_t N, uint32_t K,
                                uint32_t group, uint64_t seed, float eps, int sign, void* w_eff_dev,
                                void* stream);

/*
 * NormalFloat-4 blocks (the quantizer of the text-to-image experiment, Sec. 4.3): a block of 64
 * consecutive input features of a row shares one scale (its absmax) and each weight is the index u
 * of one of the 16 NormalFloat-4 levels in [-1, 1]:  W[n,k] = s[n, k/64] * level[u[n,k]], and a
 * perturbed pass uses (s + sign*eps*z)[n, k/64] (Eq. 4-5 with wbar = level[u]).
 *   q_dev: uint8 [N, K/2], index of even k in the low nibble; s_dev: bf16 [N, K/64];
 *   z as for qzo_dequant_gemm: counter (row_base + n, g/8), stream 0.
 * qzo_nf4_expand writes the perturbed scales (se_dev, fp32 [N, K/64], one fma each) and the perturbed
 * matrix (w_dev, bf16 [N,K], the fp32 product se * level rounded to nearest even).
 * qzo_nf4_gemm does the same into scratch_dev (qzo_nf4_scratch_bytes(N, K) bytes, 256-byte aligned,
 * contents undefined afterwards) and then Y = X W^T with the plain bf16 GEMM: x_dev bf16 [M,K],
 * y_dev bf16 [M,N].  The table lookup is done once per weight and pass, not once per token tile.
 * block must be 64, K a positive multiple of 128, N a multiple of 8, pointers 16-byte aligned.
 */
qzo_status qzo_nf4_expand(const void* q_dev, const void* s_dev, uint32_t row_base, uint32_t N,
                          uint32_t K, uint32_t block, uint64_t seed, float eps, int sign,
                          float* se_dev, void* w_dev, void* stream);
qzo_status qzo_nf4_scratch_bytes(uint32_t N, uint32_t K, uint64_t* out);
qzo_status qzo_nf4_gemm(const void* x_dev, const void* q_dev, const void* s_dev, uint32_t row_base,
                        uint32_t M, uint32_t N, uint32_t K, uint32_t block, uint64_t seed, float eps,
                        int sign, void* y_dev, void* scratch_dev, uint64_t scratch_bytes,
                        void* stream);

/*
 * Expand-then-multiply for int4 groups (Eq. 4-5) on a single linear.
 * qzo_int4_expand, the first stage: the perturbed scales se = s + sign*eps*z (se_dev, fp32 [N, K/128],
 * one fma each) and the perturbed weight matrix (w_dev, bf16 [N,K]) =
 * se[n, g(k)] * (u[n,k] - zp[n, g(k)]) rounded once to bf16.  zp_dev may be null (every zero-point 8:
 * the symmetric format).  g_idx_dev may be null (g(k) = k / 128) or point to int32 [K], the group of
 * every input column (activation reordering of the Sec. 4.1 checkpoints; values outside 0 .. K/128 - 1
 * are clamped); the noise stays per (row, group).  Other operands as for qzo_dequant_gemm_zp; without
 * g_idx the result has the same bits as the fused kernel's weight tile.
 * qzo_int4_gemm_expanded: the same into scratch_dev (qzo_int4_scratch_bytes(N, K) bytes, 256-byte
 * aligned, contents undefined afterwards), then Y = X W^T with the plain bf16 GEMM (x_dev bf16 [M,K],
 * y_dev bf16 [M,N]); the only GEMM entry point that takes g_idx.
 */
qzo_status qzo_int4_expand(const void* q_dev, const void* s_dev, const void* zp_dev,
                           const int32_t* g_idx_dev, uint32_t row_base, uint32_t N, uint32_t K,
                           uint32_t group, uint64_t seed, float eps, int sign, float* se_dev,
                           void* w_dev, void* stream);
qzo_status qzo_int4_scratch_bytes(uint32_t N, uint32_t K, uint64_t* out);
qzo_status qzo_int4_gemm_expanded(const void* x_dev, const void* q_dev, const void* s_dev,
                                  const void* zp_dev, const int32_t* g_idx_dev, uint32_t row_base,
                                  uint32_t M, uint32_t N, uint32_t K, uint32_t group, uint64_t seed,
                                  float eps, int sign, void* y_dev, void* scratch_dev,
                                  uint64_t scratch_bytes, void* stream);

/* How a model's int4 linears (quant 0 and 2) run.  mode 0 (default): by size; a linear [N,K] with at
 * least 2300 + 3.3e10 / (N K) tokens in a pass (2950 for 12288 x 4096) has its perturbed weights first
 * written out as a bf16 matrix in the workspace (same bits as the fused kernel's weight tile) and multiplied
 * by the plain bf16 GEMM, with fewer the fused dequantizing GEMM runs (below the break-even an expansion
 * costs more than the fused kernel's extra work).  mode 1: always the fused kernel.  mode 2: always expand-then-multiply.
 * A field of the model; call it before qzo_workspace_bytes (the workspace layout depends on it).
 * QZO_ERR_ARG for another mode, QZO_ERR_UNSUPPORTED for a model whose format is not int4. */
qzo_status qzo_model_set_int4_path(qzo_model* m, int mode);

/* Inspection: the second stage of the expand-then-multiply paths on its own, Y = X W^T with a plain
 * bf16 weight matrix w_dev [N,K] (x_dev bf16 [M,K], y_dev bf16 [M,N], fp32 accumulation, no epilogue).
 * pipe: 0 or 1, operand tiles staged through registers (compiler's / explicit issue order); 2, both
 * operand tiles loaded from memory straight into the LDS (no staging registers; the one the models use).  K a positive multiple of 128, N a multiple of 8, pointers
 * 16-byte aligned, M*K, N*K and M*N below 2^30 elements. */
qzo_status qzo_debug_bf16_gemm(const void* x_dev, const void* w_dev, uint32_t M, uint32_t N, uint32_t K,
                               int pipe, void* y_dev, void* stream);

/* Measurement aid, not part of the method: one 512-thread workgroup per compute unit, each
 * wavefront issuing iters x 16 v_mfma_f32_32x32x16_bf16 (32768 flop each) on register operands
 * that are all zero (random_operands = 0) or pseudo-random bf16 values, with no memory traffic.
 * Timed by the caller on `stream`, it gives the bf16 MFMA rate the board sustains under its
 * own clock and power management: flop = *workgroups_out * 8 * 16 * 32768 * iters.
 * sink_dev: fp32 [*workgroups_out * 512] device scratch (at least 512 * 512 floats are
 * enough for any device), overwritten.  iters in 1 .. 2^20. */
qzo_status qzo_debug_mfma_rate(uint32_t iters, int random_operands, float* sink_dev,
                               uint32_t* workgroups_out, void* stream);

/* qzo_forward_loss that also copies the final normalised hidden states (the lm_head's
 * input, bf16 [batch*seq, d_model]) to hidden_dev. */
qzo_status qzo_debug_forward(qzo_model* m, const int32_t* tokens_dev, uint32_t batch, uint32_t seq,
                             uint64_t seed, float eps, int sign, void* workspace_dev,
                             uint64_t workspace_bytes, float* loss_dev, void* hidden_dev,
                             void* stream);

/*
 * Measurement hooks (for benchmarks; not part of the method).  After
 * qzo_profile_begin(max_records) every kernel launch of qzo_forward_loss /
 * qzo_step is bracketed by a pair of HIP events recorded on the call's stream
 * until max_records launches have been seen.  qzo_profile_collect stops the
 * recording, waits for the recorded events and returns, for one kernel class,
 * the summed elapsed milliseconds, the number of launches and the summed
 * algorithmic work (flops for 0..2, bytes for 3).  Classes: 0 = perturbed
 * W4A16 GEMM, 1 = lm_head GEMM + cross-entropy partials, 2 = attention,
 * 3 = scale update, 4 = embedding and the joint mode's kernels, 5 = weight expansion (bytes:
 * packed weights in + bf16 out).  Host pointers.  Not thread-safe.
 * qzo_profile_stride(n): from the next qzo_profile_begin on only every n-th launch of each class is
 * bracketed (the first, the n+1-th, ...), which keeps the cost of the events (a few microseconds of
 * GPU time per bracketed launch) out of a timed run; launches, time and work then cover the bracketed
 * launches only.  A layer's four linears have different shapes: use a stride that is odd.  Default 1.
 */
qzo_status qzo_profile_stride(uint32_t stride);
qzo_status qzo_profile_begin(uint32_t max_records);
qzo_status qzo_profile_collect(uint32_t kind, double* total_ms, uint64_t* launches, double* work);

const char* qzo_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* QZO_H_ */
