/*
 * mslt.h -- C ABI of the MSLT stage-step library for AMD MI355X (gfx950).
 *
 * One training step of a stage of Multi-Stage Layerwise Training (paper Section 3.2):
 * the bottom `frozen_layers` encoder layers of a BERT stack, trained in earlier stages, run
 * forward only and keep no intermediates; the `trainable_layers` layers above them and the
 * output layer (masked-LM head) run forward and backward and are the only tensors that get
 * gradients and an optimizer update (Section 3.1, last paragraph; Figure 1).  The embedding
 * block with the word matrix shared between input and output is trained only when nothing is
 * frozen -- the first stage and the final joint retraining (Section 3.2).
 *
 * Conventions
 *   - Every function returns 0 on success and a negative mslt_status on error; the message of
 *     the last error of the calling thread is available from mslt_last_error().  A call that
 *     fails validation of its arguments (MSLT_ERR_ARG, MSLT_ERR_STATE) enqueues no GPU work and
 *     leaves every arena untouched.  A step refused for its batch content (MSLT_ERR_DATA) leaves
 *     parameters, gradients of earlier steps' tensors, moments and step counts untouched, but it
 *     has used the workspace arena and ends the validity of the previous step's results: the
 *     gradient read-back, the update and both debug read-backs need a new successful step.
 *   - The library never allocates or frees device memory.  The caller (normally PyTorch) owns
 *     four device arenas whose sizes mslt_query_sizes() reports, and a HIP stream; all GPU work
 *     is ordered with that stream: part of a step runs on a second stream the model creates
 *     (default priority), which forks from the caller's stream and joins it again by events
 *     inside the same call, so work the caller enqueues on its stream before or after a call is
 *     ordered with all of the call's work.  Host memory passed in is read or written before the
 *     call returns.  "DEVICE" / "HOST" below say where a pointer must live.
 *   - Weight matrices are [out, in] row-major fp32 in the canonical tensor order reported by
 *     mslt_tensor_table(): embedding block, encoder layers bottom to top, head.
 *   - precision 0: fp32 storage and arithmetic everywhere.  precision 1: bf16 activations and
 *     bf16 shadow copies of the weight matrices feeding MFMA, fp32 accumulation, fp32 softmax /
 *     LayerNorm / GELU / cross-entropy internals, fp32 gradients, master weights and optimizer
 *     state.
 *   - Calls on one model must not overlap; they are not thread-safe.
 */
#ifndef MSLT_H
#define MSLT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mslt_model mslt_model; /* opaque host object; owns no device memory */

enum mslt_status {
  MSLT_OK = 0,
  MSLT_ERR_ARG = -1,      /* null pointer, bad shape, bad layer split, size mismatch */
  MSLT_ERR_STATE = -2,    /* call order: update / get_grads without a successful step */
  MSLT_ERR_DATA = -3,     /* batch content: id out of range, no predicted position, too many */
  MSLT_ERR_HIP = -4,      /* a HIP runtime call failed */
  MSLT_ERR_NONFINITE = -5 /* the step ran but the loss is not finite */
};

typedef struct {
  int n_layers_max;    /* encoder layers the arenas hold (12 Base, 24 Large: Section 4.1) */
  int hidden;          /* H; multiple of 4, at most 2048 */
  int n_heads;         /* H / n_heads = head width, at most 128 */
  int ffn;             /* F */
  int vocab;           /* V */
  int max_pos;         /* rows of the position table; seq <= max_pos */
  int type_vocab;      /* rows of the token-type table */
  int max_batch;       /* largest batch a step may bring */
  int max_seq;         /* largest sequence length a step may bring */
  int max_predictions; /* largest number of predicted positions per step; 0 = max_batch*max_seq */
  int precision;       /* 0 fp32, 1 bf16 compute with fp32 master */
  float ln_eps;        /* LayerNorm epsilon (1e-12) */
  float mask_bias;     /* added to the scores of padded keys (-10000) */
  int layers_per_group; /* 0 or 1: every layer has its own parameters (BERT).  n > 1: the grouped ALBERT
                          variant of Section 3.3 - each run of n consecutive layers shares one parameter set
                          ("layer g" in the tensor table is the set of group g; there are n_layers_max / n sets),
                          the gradients of a set are the sums over its n applications, and the layer counts of
                          mslt_stage_step / mslt_train_step / mslt_grow must be whole groups */
  int with_nsp;         /* 1: the model also has BERT's next-sentence head (Section 4.1 keeps both objectives):
                          pooler.w [H,H], pooler.b [H] (dense + tanh on the first token of every sequence) and
                          nsp.w [2,H], nsp.b [2] after the masked-LM head in the tensor table; they train in every
                          stage, the step's loss is the sum of the two mean cross-entropies, and every step's batch
                          must bring nsp_labels */
  int max_trainable_layers; /* largest number of layers one step may train; 0 = n_layers_max.  Only trainable layers keep
                          intermediates for the backward pass (Section 3.2: the layers below only take part in the
                          forward computation), so the workspace holds that many per-layer stashes: a model that
                          only ever runs stages of N/k layers can be given N/k here (BERT-Large, 24 layers, batch
                          32 x 512: 6 instead of 24 saves about 10 GB); a step that asks for more is refused */
} mslt_config;

/* One masked-LM batch.  DEVICE pointers to int32 arrays of batch*seq entries, row-major
 * [batch][seq], owned by the caller and valid until the step's stream work has finished.
 * attn_mask: 1 token, 0 padding.  labels: original id at predicted positions, -100 elsewhere. */
typedef struct {
  const int32_t* input_ids;
  const int32_t* token_type_ids;
  const int32_t* attn_mask;
  const int32_t* labels;
  int batch;
  int seq;
  const int32_t* nsp_labels; /* DEVICE, [batch], 0 or 1; read only by a model with with_nsp = 1, else may be null */
} mslt_batch;

/* Optimizer of the update (Section 4.1: LAMB, lr 0.00088; Section 5 also names Adam).
 * u = mhat/(sqrt(vhat)+eps) + weight_decay*w (decay on matrices and embedding tables only).
 * kind 0 Adam: w -= lr*u.  kind 1 LAMB: w -= lr*(|w|/|u|)*u per logical tensor (ratio 1 if a
 * norm is 0).  bias_correction != 0 divides m, v by (1-beta^t), t counted per tensor. */
typedef struct {
  int kind;
  float lr, beta1, beta2, eps, weight_decay;
  int bias_correction;
} mslt_opt;

typedef struct {
  char name[32];  /* "emb.word", "layer3.wq", "head.b_out", ... */
  int layer;      /* encoder layer index, -1 embedding block, -2 head */
  int rows, cols; /* logical shape; cols = 1 for vectors */
  int decays;     /* 1 if weight decay applies */
  size_t offset;  /* element offset inside the parameter / gradient / moment arenas */
  size_t count;   /* rows*cols */
} mslt_tensor_desc;

/* Arena sizes in bytes for a configuration.  param_bytes: fp32 master weights.  grad_bytes:
 * fp32 gradients (same offsets).  opt_state_bytes: first and second moments.  workspace_bytes:
 * bf16 shadows, activations, the stash of the trainable layers, head buffers, reduction scratch.
 * HOST pointers; any may be null. */
int mslt_query_sizes(const mslt_config* cfg, size_t* param_bytes, size_t* grad_bytes, size_t* opt_state_bytes,
                     size_t* workspace_bytes);

/* Creates a model over caller-owned DEVICE arenas (each at least the queried size, 256-byte
 * aligned) and a HIP stream (hipStream_t passed as void*, null = default stream).  Zero-fills all
 * four arenas on the stream: parameters and optimizer state start at zero, step counts at 0.
 * *out is a HOST object to be released with mslt_destroy(). */
int mslt_init_model(const mslt_config* cfg, void* param_arena, void* grad_arena, void* opt_arena, void* workspace,
                    void* hip_stream, mslt_model** out);

/* Canonical tensor list.  *out points to an array of *n descriptors owned by the model. */
int mslt_tensor_table(const mslt_model* m, int* n, const mslt_tensor_desc** out);

/* Loads all parameters from a packed HOST fp32 array in canonical order (n_floats = sum of
 * counts) and rebuilds the bf16 shadows.  Blocks until the copy is done. */
int mslt_load_params(mslt_model* m, const float* host_fp32, size_t n_floats);

/* Reads all parameters back into a packed HOST fp32 array in canonical order.  Blocks. */
int mslt_get_params(const mslt_model* m, float* host_fp32_out, size_t n_floats);

/* One stage step (Section 3.2): forward through layers [0, frozen+trainable), masked-LM loss,
 * backward through the head and the top `trainable_layers` layers only.  Layers above
 * frozen+trainable are not executed (the stack of an earlier stage is shallower).
 * Requirements: trainable_layers >= 1 (and <= max_trainable_layers when that is set), frozen_layers >= 0,
 * frozen+trainable <= n_layers_max,
 * train_embeddings may be 1 only if frozen_layers == 0, batch <= max_batch, seq <= max_seq,
 * at least one and at most max_predictions predicted positions, ids inside their tables
 * (checked on the device; the encoder forward is queued meanwhile, reading the tables with clamped
 * indices, and nothing that a later call can observe is written before the verdict; violations
 * return MSLT_ERR_DATA).
 * Gradients of exactly the trainable tensors are left in the gradient arena.  *loss_out (HOST)
 * receives the mean loss over predicted positions; the call waits for the stream for this. */
int mslt_stage_step(mslt_model* m, int frozen_layers, int trainable_layers, int train_embeddings,
                    const mslt_batch* batch, float* loss_out);

/* Number of floats mslt_get_grads() will write for the last successful step. */
int mslt_grad_count(const mslt_model* m, size_t* n_floats);

/* Gradients of the last step's trainable tensors, packed in canonical order, to HOST. Blocks. */
int mslt_get_grads(const mslt_model* m, float* host_fp32_out, size_t n_floats);

/* Applies the optimizer to exactly the tensors that received gradients in the last step
 * (Section 3.2: only the new top layers and the output layer are updated; everything is updated
 * in the first stage and in retraining) and refreshes their bf16 shadows.  Frozen tensors, their
 * moments and step counts are not touched.  Enqueues work only; does not block.  A second call
 * without a new step is an error.  After a step that returned MSLT_ERR_NONFINITE the call is
 * accepted but its kernels change nothing (they test that step's loss on the device). */
int mslt_apply_update(mslt_model* m, const mslt_opt* opt);

/* mslt_apply_update() for callers that cannot allocate or hand over scratch memory of their own
 * choosing (code under HIP graph capture, tight serving-style loops, harnesses that forbid hipMalloc):
 * same update, same results bit for bit, but the only scratch the update needs (LAMB's per-chunk
 * partial sums and per-tensor trust ratios) lives in a device array inside the library (266 240 bytes
 * per GPU, held until the process ends) instead of the workspace arena.  The call allocates and frees
 * nothing.  Limits: at most 32768 optimizer chunks of 16384 elements (about 536 M parameters) and
 * 1024 tensors in the model's tensor table; larger models get MSLT_ERR_ARG and nothing is enqueued.
 * All models on one GPU share that array and it keeps the previous call's contents (every value read
 * is written earlier in the same call, so nothing has to be cleared): calls that overlap in time on
 * one GPU, from different models or streams, race.  Enqueues work only; does not block. */
int mslt_apply_update_static(mslt_model* m, const mslt_opt* opt);

/* One training step of a stage in one call: mslt_stage_step() followed by mslt_apply_update()
 * (Sections 3.1 and 3.2), with the same requirements, results and error codes as the two calls
 * made one after the other.  The update is queued right behind the step, before the host has
 * seen the loss, so the device does not idle between the two; on the device it does nothing when
 * the loss is not finite, and the call then returns MSLT_ERR_NONFINITE with the parameters, the
 * moments and the step counts unchanged.  *loss_out (HOST) as in mslt_stage_step(); the call
 * waits for the stream.  The gradients are consumed: mslt_get_grads() needs a new
 * mslt_stage_step(). */
int mslt_train_step(mslt_model* m, int frozen_layers, int trainable_layers, int train_embeddings,
                    const mslt_batch* batch, const mslt_opt* opt, float* loss_out);

/* Dropout for the steps that follow (BERT's dropout, which Section 4.1 adopts by reference:
 * probability 0.1 on the embedding output, the attention probabilities, the attention output and
 * the feed-forward output, in frozen and trainable layers alike).  p in [0, 1); p = 0 (the state
 * after mslt_init_model) switches it off.  The keep decisions are counter-based and reproducible:
 * element e (C-order index in the dropped tensor) of site s (0 embedding [T,H], 1 attention
 * probabilities [B,heads,S,S], 2 attention output [T,H], 3 feed-forward output [T,H]) of layer l is
 * kept iff bits 16*(e%4) .. +15 of mix(key + (e/4) * 0x9E3779B97F4A7C15) are >= round(p * 65536),
 * where mix is the SplitMix64 output function and key = mix(seed ^ mix(((step << 20) | (l << 4) | s)
 * + 0x9E3779B97F4A7C15)); kept values are scaled by 1 / (1 - p).  The caller advances `step`
 * (below 2^44) from one training step to the next; the same (seed, step) repeats the same masks.
 * The hidden size must be a multiple of 4. */
int mslt_set_dropout(mslt_model* m, float p, uint64_t seed, uint64_t step);

/* Predicted positions (ascending flat index b*seq+s) and their labels as found by the last
 * step, to HOST arrays of at least max_predictions entries; *m_out = their number.  Blocks. */
int mslt_debug_masked(const mslt_model* m, int32_t* pos_out, int32_t* label_out, int* m_out);

/* Output of the frozen prefix of the last step (the input of the lowest trainable layer;
 * the embedding output if nothing was frozen), batch*seq*hidden values widened to fp32, to
 * HOST.  Blocks.  Valid until the next step. */
int mslt_debug_prefix_output(const mslt_model* m, float* host_fp32_out, size_t n_floats);

/* Stack growth between stages (Section 3.2): layer n_present+i becomes a copy of layer
 * n_present-n_new+i, i = 0..n_new-1 (parameters and shadows); the new layers' moments are
 * zeroed and their step counts reset.  Enqueues work only. */
int mslt_grow(mslt_model* m, int n_present, int n_new);

/* Measurement aid (Section 4 reports wall-clock time only; this gives the per-kernel view).
 * While enabled, every group of launches of one kernel class is bracketed by two HIP events on
 * the model's stream.  mslt_profile_read() waits for the stream, adds up per class the elapsed
 * time, launch groups, algorithmic FLOPs and algorithmic HBM bytes since the last read into
 * `out` (HOST array of at least 16 entries; *n = entries written) and clears the record.
 * Event recording costs a few microseconds per launch: keep it off when timing whole steps. */
typedef struct {
  char name[24];
  int launches;
  double ms, flops, bytes;
} mslt_profile_entry;
int mslt_profile_enable(mslt_model* m, int on);
int mslt_profile_read(mslt_model* m, mslt_profile_entry* out, int cap, int* n);

/* Test and measurement aid for the matrix products the step is made of (Sections 3.1 and 3.2 name
 * the layers; their linear maps are these products): C[M,N] = sum_k A(m,k) B(n,k) on DEVICE operands
 * through one chosen kernel, enqueued on hip_stream (hipStream_t as void*, null = default stream).
 * A and B are bf16 (2 bytes per element, round to nearest even); a_kcontig != 0: A(m,k) = A[m*K + k],
 * else A[k*M + m]; the same for B with n and N.  C is row-major [M,N], bf16, or fp32 when out_f32 != 0.
 * kernel 0: guarded SIMT kernel (any shape).  kernel 1: 128-wide MFMA kernel, tile_m 0 (chosen by
 * shape), 128 or 256; M % 128 == 0, N % 128 == 0, K % 64 == 0.  kernel 2: large-tile kernel fed by
 * direct global-to-LDS loads, tile_m x tile_n one of 256x256, 256x128, 128x256, 128x128, ring stage
 * tile_k 64 (or 32, not for 128x128); M % tile_m == 0, N % tile_n == 0, K % tile_k == 0.  splitk > 1
 * (kernels 1 and 2) splits the contraction over workgroups and needs `partials`, DEVICE scratch of at
 * least splitk*M*N*4 bytes (partial_bytes says how large it is).  Returns MSLT_ERR_ARG for a shape or
 * choice the kernel does not take; nothing is enqueued then.  Does not block. */
int mslt_debug_gemm(void* hip_stream, const void* A, const void* B, void* C, int M, int N, int K, int a_kcontig,
                    int b_kcontig, int out_f32, int kernel, int tile_m, int tile_n, int tile_k, int splitk,
                    void* partials, size_t partial_bytes);

/* Waits until all work enqueued on the model's stream has finished. */
int mslt_sync(const mslt_model* m);

int mslt_destroy(mslt_model* m);

/* Message of the calling thread's last error ("" if none). */
const char* mslt_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MSLT_H */
