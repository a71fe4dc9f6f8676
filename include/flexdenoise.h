/* flexdenoise.h -- C ABI of the MI355X-native denoising path.
 *
 * What the library computes.  FlexCache (arXiv 2501.04012) serves a text-to-video
 * request either from Gaussian noise or, on a cache hit, from the stored latent of
 * an earlier request's step k: the stored latent is set as the input and generation
 * proceeds from the next step (Sec. 2.2 "Caching for Diffusion Models"; Sec. 3.2
 * "Cache lookup"; Sec. 4.2.2: a step-10 cache lets the request proceed from the
 * 11th step).  A denoising step takes the current latent and the prompt embedding,
 * predicts the noise and removes it; steps are sequential and dominate a request's
 * run time (Sec. 2.1 "Diffusion Model"; Sec. 6.2.1 "Performance Breakdown").  This
 * library is that step, and the loop over the remaining N-k steps, for a latent
 * video diffusion transformer.
 *
 * The paper fixes neither the network nor the sampler constants; the network here
 * is a pre-LN adaLN diffusion transformer in two video forms (attn_mode), the
 * sampler is deterministic DDIM (eta = 0) on a linear-beta schedule with
 * classifier-free guidance.
 *
 * Conventions for every call
 *   - returns an int status: FC_OK (0) or a negative FC_ERR_*; never throws, never
 *     aborts, never prints.  fc_last_error() gives a per-thread message.
 *   - "dev" pointers are HIP device pointers on the current device, "host"
 *     pointers are ordinary host memory.  The caller owns every buffer it passes;
 *     the library owns the fc_model and the device copy of the weights.
 *   - work is enqueued on the given hipStream_t (passed as void*; NULL = the
 *     default stream) and is NOT synchronised: the caller synchronises the stream.
 *   - nothing allocates device memory after fc_model_set_weights(); all scratch
 *     comes from the caller's workspace.
 *   - one fc_model may be used by one host thread at a time.  Results are
 *     run-to-run bitwise deterministic (no atomics in any reduction).
 */
#ifndef FLEXDENOISE_H
#define FLEXDENOISE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fc_model fc_model; /* opaque, library-owned */

enum {
  FC_OK = 0,
  FC_ERR_NULL = -1,        /* a required pointer is NULL */
  FC_ERR_SHAPE = -2,       /* inconsistent configuration (divisibility, sizes) */
  FC_ERR_RANGE = -3,       /* step / k / batch outside its range */
  FC_ERR_WORKSPACE = -4,   /* workspace smaller than fc_workspace_bytes() */
  FC_ERR_DEVICE = -5,      /* a HIP call failed */
  FC_ERR_UNSUPPORTED = -6, /* a combination the library does not implement (eta != 0 with the Euler
                              sampler, more than 256 frames in a cache entry, a forced kernel whose
                              shape conditions are not met) */
  FC_ERR_STATE = -7        /* weights not set yet */
};

enum { FC_ATTN_FACTORIZED_CROSS = 0, /* spatial attn, temporal attn, text cross-attn per block */
       FC_ATTN_FULL3D_CONCAT = 1 };  /* one attention over [text ; video] tokens per block */
enum { FC_F32 = 0,   /* fp32 weights, activations and arithmetic */
       FC_BF16 = 1 };/* bf16 weights/activations on MFMA, fp32 accumulation, fp32 residual stream */

/* Model shape.  Latent is [frames, height, width, channels]; patches are
 * patch x patch in space (temporal patch 1), so a frame has
 * S = (height/patch)*(width/patch) tokens and the video N = frames*S tokens in
 * (t, h', w') row-major order.  hidden % heads == 0, hidden % 4 == 0, hidden <= 4096,
 * height % patch == 0, width % patch == 0, t_embed_dim even. */
typedef struct {
  int32_t frames, height, width, channels, patch;
  int32_t hidden, heads, mlp_dim, depth;
  int32_t text_len, text_dim, t_embed_dim;
  int32_t attn_mode; /* FC_ATTN_* */
  int32_t dtype;     /* FC_F32 or FC_BF16 */
  float ln_eps;      /* LayerNorm epsilon (affine-free, biased variance) */
  int32_t text_adaln;/* FC_ATTN_FULL3D_CONCAT only: 1 = the text rows are modulated and gated by a
                        set of vectors of their own (variant); 0 = one set for all rows */
} fc_model_config;

/* Sampler.
 * FC_SAMPLER_DDIM (eps-prediction): beta_i linear from beta_start to beta_end over
 * train_steps; the num_steps sampling timesteps are tau_j = j*(train_steps/num_steps),
 * visited in descending order; step s (1-based) maps t = tau_{N-s} to tau_{N-s-1}, the
 * last step to abar_prev = 1.  eta in 0..1: 0 is the deterministic update; eta > 0 adds
 * sigma z with sigma = eta sqrt((1-abar_prev)/(1-abar_t)) sqrt(1 - abar_t/abar_prev) and
 * keeps sqrt(1 - abar_prev - sigma^2) eps (the paper changes the denoising seed after a
 * retrieval, which needs a sampler that draws noise).  z is a function of (seed,
 * request index in the batch, step, element): Philox4x32-10 with counter (i/4 low word,
 * i/4 high word, step, request) and key (seed low, seed high) gives elements 4(i/4) ..
 * +3; an output word w becomes u = ((w >> 8) + 0.5) 2^-24; words (0, 1) and (2, 3) are
 * Box-Muller pairs (sqrt(-2 ln u_a) cos(2 pi u_b), ... sin(2 pi u_b)).
 * FC_SAMPLER_FLOW_EULER (variant; the network output is the velocity noise - x0 of the
 * straight path x_sigma = (1 - sigma) x0 + sigma noise): sigma_j = j/N; step s goes from
 * sigma_{N-s+1} to sigma_{N-s}, x <- x + (sigma_{N-s} - sigma_{N-s+1}) v, the network is
 * evaluated at t = sigma_{N-s+1} * train_steps (train_steps % num_steps == 0 required);
 * beta_* are not used and eta must be 0.  The resume loop is the same for both. */
#define FC_SAMPLER_DDIM 0
#define FC_SAMPLER_FLOW_EULER 1
typedef struct {
  int32_t train_steps;
  float beta_start, beta_end;
  int32_t num_steps;
  float guidance_scale; /* used only when null_cond != NULL */
  float eta;
  int32_t sampler;      /* FC_SAMPLER_* */
  uint64_t seed;        /* key of the noise when eta > 0 */
} fc_schedule;

/* Create a model for `cfg` on the current device.  *out receives the handle.
 * Errors: FC_ERR_NULL, FC_ERR_SHAPE, FC_ERR_DEVICE. */
int fc_model_create(const fc_model_config* cfg, fc_model** out);

/* Number of floats fc_model_set_weights() expects for this model. */
int fc_model_weight_count(const fc_model* m, size_t* out);

/* Upload all parameters.  host_blob (host, fp32, little-endian) is the
 * concatenation, in this order, of row-major tensors with linear weights stored
 * [in, out] (y = x W + b):
 *   t_w1[te,D] t_b1[D] t_w2[D,D] t_b2[D]   timestep MLP on the sinusoid
 *   y_w[dt,D] y_b[D]                      text projection
 *   p_w[p*p*C,D] p_b[D]                   patch embedding (patch feature order dh,dw,c)
 *   per block, FACTORIZED_CROSS:
 *     mod_w[D,9D] mod_b[9D]  (shift,scale,gate) x (spatial, temporal, mlp)
 *     sp_qkv_w[D,3D] b  sp_proj_w[D,D] b  tm_qkv_w[D,3D] b  tm_proj_w[D,D] b
 *     x_q_w[D,D] b  x_kv_w[D,2D] b  x_proj_w[D,D] b
 *     fc1_w[D,M] b  fc2_w[M,D] b
 *   per block, FULL3D_CONCAT:
 *     mod_w[D,6D] mod_b[6D]  (shift,scale,gate) x (attn, mlp); with text_adaln [D,12D], [12D]:
 *                            the video rows' six chunks, then the text rows' six
 *     qkv_w[D,3D] b  proj_w[D,D] b  fc1_w[D,M] b  fc2_w[M,D] b
 *   f_mod_w[D,2D] f_mod_b[2D]  (shift,scale) of the final layer
 *   f_w[D,p*p*C] f_b[p*p*C]
 * qkv columns are [q | k | v], each split into `heads` consecutive groups.
 * The blob is copied (and rounded to bf16, nearest-even, for FC_BF16); the caller
 * may free it on return.  This call allocates device memory and synchronises.
 * Errors: FC_ERR_NULL, FC_ERR_SHAPE (n_floats mismatch), FC_ERR_DEVICE. */
int fc_model_set_weights(fc_model* m, const float* host_blob, size_t n_floats);

/* Free the model and its device memory.  NULL is accepted. */
int fc_model_destroy(fc_model* m);

/* Bytes of device workspace a step/resume call needs for `batch_requests`
 * requests, with (use_cfg != 0) or without a guidance pair. */
int fc_workspace_bytes(const fc_model* m, int32_t batch_requests, int32_t use_cfg, size_t* out);

/* One denoising step (Sec. 2.1): latent <- DDIM update of latent with the guided
 * noise estimate, for the step-th (1-based) of sched->num_steps steps.
 *   latent     dev, fp32 [R, frames, height, width, channels], updated in place
 *   cond       dev, fp32 [R, text_len, text_dim], prompt embeddings
 *   null_cond  dev, fp32 [text_len, text_dim] shared 'empty prompt' embedding, or
 *              NULL for no classifier-free guidance
 *   eps_out    dev, fp32, same shape as latent, receives the (guided) noise
 *              estimate; may be NULL
 * Errors: FC_ERR_NULL, FC_ERR_STATE, FC_ERR_RANGE (step not in 1..N, R < 1,
 * eta outside 0..1), FC_ERR_UNSUPPORTED (eta != 0 with the Euler sampler),
 * FC_ERR_WORKSPACE, FC_ERR_DEVICE. */
int fc_denoise_step(fc_model* m, float* latent, const float* cond, const float* null_cond,
                    const fc_schedule* sched, int32_t step, int32_t batch_requests,
                    float* eps_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Cache-hit resume (Sec. 2.2; Sec. 3.2 "Cache lookup"; Sec. 4.2.2): `latent`
 * holds the stored latents after step k; runs steps k+1 .. N in place.  k = 0 is
 * a full generation from noise, k = N returns at once.  All R requests share k.
 * Work that does not depend on the timestep (text projection, cross-attention
 * keys/values) is done once per call.  Arguments and errors as fc_denoise_step,
 * with FC_ERR_RANGE for k outside 0..N. */
int fc_denoise_resume(fc_model* m, float* latent, const float* cond, const float* null_cond,
                      const fc_schedule* sched, int32_t k, int32_t batch_requests,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* fc_denoise_resume that also hands out intermediate latents: after step export_steps[e]
 * (ascending, each in k+1 .. N; host array) the latents of all R requests are copied to
 * export_dst[e] (host array of dev pointers, each R*T*H*W*C floats) in stream order, without
 * a host wait.  These are the latents a cache inserts for the key steps between the step
 * that was hit and the last cached step (Sec. 4.2.4 "Cache Operations", Insertion).
 * n_export = 0 is fc_denoise_resume.  Errors as fc_denoise_resume, FC_ERR_RANGE for steps
 * outside k+1 .. N or not ascending. */
int fc_denoise_resume_ex(fc_model* m, float* latent, const float* cond, const float* null_cond,
                         const fc_schedule* sched, int32_t k, int32_t batch_requests,
                         int32_t n_export, const int32_t* export_steps, float* const* export_dst,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* The four coefficients of a step, as the update kernel receives them (computed in
 * double, rounded to float), for x0 = (x - c1 e) / c0, x <- c2 x0 + c3 e:
 * DDIM: out4 = { sqrt(abar_t), sqrt(1-abar_t), sqrt(abar_prev), sqrt(1-abar_prev) };
 * with eta > 0 the fourth is sqrt(1 - abar_prev - sigma^2);
 * Euler: { 1, 0, 1, sigma_next - sigma }.  *t_out = timestep the network is evaluated
 * at.  Host only. */
int fc_schedule_coefficients(const fc_schedule* sched, int32_t step, float* out4, int32_t* t_out);

const char* fc_status_string(int status);
const char* fc_last_error(void);

/* ---- per-kernel timing.  While enabled, every launch group of a step is bracketed by a
 * HIP event pair recorded on the call's stream.  fc_profile_read() waits for the
 * recorded events, adds the elapsed milliseconds and the number of brackets per
 * category into ms_out / launches_out (host arrays of n >= fc_profile_categories()
 * entries) and clears the record.  Categories are named by
 * fc_profile_category_name(i).  fc_profile_categories() returns the count, not a status.
 * fc_profile_select() restricts the brackets to one category (-1: all, the default), so
 * that a timed run carries the events of the kernel of interest only. */
/* The category names in index order, separated by single spaces. */
#define FC_PROFILE_CATEGORY_NAMES                                                          \
  "gemm_qkv gemm_proj gemm_fc1 gemm_fc2 gemm_other attn_spatial attn_temporal attn_cross " \
  "attn_full3d ln_modulate patch_embed timestep_modulation cfg_ddim other"
int fc_profile_enable(fc_model* m, int32_t enable);
int fc_profile_select(fc_model* m, int32_t category);
int fc_profile_categories(void);
const char* fc_profile_category_name(int32_t i);
int fc_profile_read(fc_model* m, int32_t n, double* ms_out, int64_t* launches_out);

/* ---- restoring a cached latent: what produces the `latent` argument of a resume.
 * Latents are f32 [frames, H, W, C]; a "frame" below is its H*W*C = frame_elems floats. */

/* Stitching of a decoupled hit (Sec. 4.2.2 "Video Latent Reconstruction"): out takes a
 * pixel (all `channels` values) from x_obj where the object mask is set or the background
 * mask is clear, else from x_bg.  Masks (dev): 1 bit per pixel, pixel i in bit i % 8 of
 * byte i / 8, (pixels + 7) / 8 bytes; m_bg NULL = background valid everywhere.  out may
 * be x_obj or x_bg itself.  All pointers dev. */
int fc_cache_stitch(const float* x_obj, const float* x_bg, const uint8_t* m_obj, const uint8_t* m_bg,
                    float* out, int64_t pixels, int32_t channels, void* hip_stream);

/* Expanding a compressed entry of one step (Sec. 4.1.1 decompression, Sec. 4.1.2 Eq. 1,
 * Sec. 4.3 "Cache Entry Structure"): out[t] (dev, frames x frame_elems) is built from
 * source code src[t] (host array): 0 = first (the stored first frame of the step);
 * j in 1..n_base = first + alpha * diff_base[j-1] (a common key frame); -(e+1) =
 * extra[e] (a key frame stored whole).  Repeated key frames are repeated codes.
 * first, diff_base [n_base, frame_elems], extra [n_extra, frame_elems], out: dev.
 * At most 256 frames (FC_ERR_UNSUPPORTED); FC_ERR_RANGE for a code outside the entry. */
int fc_cache_decompress(const float* first, const float* diff_base, int32_t n_base, float alpha,
                        const float* extra, int32_t n_extra, const int32_t* src, int32_t frames,
                        int64_t frame_elems, float* out, void* hip_stream);

/* Bytes of device workspace (8-byte aligned) for the two reductions below. */
size_t fc_cache_workspace_bytes(int32_t frames);

/* The coefficient of Eq. 2 (Sec. 4.1.2): alpha_out[0] (dev) = sum((keys_s - first_s) *
 * diff_base) / sum(diff_base^2) over n_base frames; first_s [frame_elems], keys_s and
 * diff_base [n_base, frame_elems], all dev.  Sums in double, fixed order (bitwise
 * repeatable). */
int fc_cache_alpha(const float* first_s, const float* keys_s, const float* diff_base, int32_t n_base,
                   int64_t frame_elems, float* alpha_out, void* workspace, size_t workspace_bytes,
                   void* hip_stream);

/* sim [frames, frames] (dev, f32) = cosine similarity of every pair of frames of
 * frames_dev [frames, frame_elems] (Sec. 4.1.1; Sec. 5 "Cache compressor"). */
int fc_cache_frame_similarity(const float* frames_dev, int32_t frames, int64_t frame_elems, float* sim,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* fc_cache_frame_similarity for callers that cannot allocate or hand over device memory of
 * their own: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same kernels and result (bit for bit); the Gram matrix sits in a 512 KB
 * device array owned by the library (one per device, held until the process ends) instead
 * of a workspace.  At most 256 frames (FC_ERR_UNSUPPORTED beyond).  Calls no hipMalloc,
 * hipFree or allocating routine.  All calls on one device share that array: two calls that
 * overlap on one device (different streams, or threads) race; calls on one stream are safe.
 * Nothing in the array needs clearing between calls.  frames_dev, sim: dev. */
int fc_cache_frame_similarity_noalloc(const float* frames_dev, int32_t frames, int64_t frame_elems,
                                      float* sim, void* hip_stream);

/* Key-frame choice of Sec. 4.1.1 on a host copy of sim: frames are visited from the last
 * to the first; an unassigned frame becomes a key frame and every unassigned frame in
 * front of it with sim >= threshold is mapped to it.  map_out[f] (host) = the key frame
 * standing for frame f.  Host only. */
int fc_cache_select_key_frames(const float* sim, int32_t frames, float threshold, int32_t* map_out);

/* ---- single operators of the step, exposed for per-kernel tests and timing.
 * All pointers dev; dtype FC_F32 -> float elements, FC_BF16 -> bfloat16 (uint16)
 * elements for every tensor marked "act". ------------------------------------- */

/* out[M,N] (act) = epilogue(A[M,K] (act) * Wt[N,K]^T (act) + bias[N] (f32)).
 * epilogue 0: bias only; 1: bias + GELU(tanh); 2: gate[N] (f32, NULL = ones) times
 * (bias added): the gated branch output whose residual add the next LayerNorm performs.
 * The network's linear layers. */
int fc_op_linear(int32_t dtype, const void* A, const void* Wt, const float* bias, const float* gate,
                 void* out, int32_t M, int32_t N, int32_t K, int32_t epilogue, void* hip_stream);

/* fc_op_linear with scratch memory lent by the caller (dev, 16-byte aligned, scratch_bytes;
 * contents undefined afterwards), as the linear layers run inside a step: when the tiles of
 * the product leave a last round that fills at most half the chip, that round's tiles are
 * split along K, their fp32 partial tiles (at most 128 tiles x 2 ranges or 64 x 4, of 256 x 256
 * floats: 64 MB) pass through the scratch and a second launch adds them in a
 * fixed order and applies the epilogue.  Too little scratch: the product runs unsplit.
 * Same result as fc_op_linear up to the order of the fp32 additions along K. */
int fc_op_linear_scratch(int32_t dtype, const void* A, const void* Wt, const float* bias, const float* gate,
                         void* out, int32_t M, int32_t N, int32_t K, int32_t epilogue, void* scratch,
                         size_t scratch_bytes, void* hip_stream);

/* Unmasked softmax(q k^T / sqrt(d)) v for G independent problems (one per
 * sequence and head).  q [G, nq, d], k [G, nk, d], v [G, nk, d], out [G, nq, d]
 * (all act).  impl 0: library's choice, 1: force the plain (non-MFMA) kernel.
 * The MFMA kernels multiply bf16(q * log2(e)/sqrt(d)): inside a step the QKV epilogue
 * produces that from fp32 with one rounding; with impl 0 this stand-alone entry has to
 * round its bf16 q a second time.  impl 2: library's choice of kernel, and q is taken to
 * hold q' = q * log2(e)/sqrt(d) already, i.e. out = softmax_2(q' k^T) v with
 * softmax_2 the softmax to base 2: exactly what a step runs. */
int fc_op_attention(int32_t dtype, const void* q, const void* k, const void* v, void* out,
                    int32_t G, int32_t nq, int32_t nk, int32_t d, int32_t impl, void* hip_stream);

/* The attention of a long sequence as a step runs it (bf16, head dim 64 or 72): q holds
 * q' = q * log2(e)/sqrt(d) as in impl 2 above, and the keys' largest Euclidean norm per problem
 * is computed first (into key_norm_scratch: dev, 32 * G floats, overwritten), which bounds
 * every score by |q'| max|k| and lets the kernel drop the running maximum where that bound
 * is close enough to the first tile's maximum (otherwise it keeps it: same result up to
 * rounding).  Key sequences too short to profit run the same kernels as fc_op_attention. */
int fc_op_attention_bounded(const void* q, const void* k, const void* v, void* out, int32_t G, int32_t nq,
                            int32_t nk, int32_t d, float* key_norm_scratch, void* hip_stream);

/* If y (act, [M,D]) is not NULL: x[M,D] (f32) <- x + y first (the pending branch output).
 * Then out[M,D] (act) = LayerNorm(x) * (1 + scale[D]) + shift[D] (shift/scale f32, both
 * NULL = plain LayerNorm); D a multiple of 4, at most 4096. */
int fc_op_layernorm_modulate(int32_t dtype, float* x, const void* y, const float* shift,
                             const float* scale, void* out, int32_t M, int32_t D, float eps,
                             void* hip_stream);

/* The same with the residual additions as a step defers them (the pre-LN block of the DiT
 * sections: x <- x + gate * branch(LayerNorm(x)), one addition per branch): up to two pending
 * branch outputs y, y2 (act, [M,D]; y2 only together with y), each with an optional per-column
 * gate (f32 [D], NULL = ones), are added in that order to the row in fp32,
 *   v = (x + gate * y) + gate2 * y2,   out = LayerNorm(v) * (1 + scale) + shift,
 * and v is written back to x only if write_x is non-zero; otherwise x is left as it is and the
 * caller passes the same y again with the next branch's output. */
int fc_op_layernorm_residual2(int32_t dtype, float* x, const void* y, const float* gate, const void* y2,
                              const float* gate2, const float* shift, const float* scale, void* out,
                              int32_t M, int32_t D, float eps, int32_t write_x, void* hip_stream);

/* Patch embedding with positions: x[b, row_off + n, :] (f32, rows of D, rows_per_b rows per
 * batch row) = patch(latent[b % R], n) . Wp[p*p*C, D] + bp[D] + pos_sp[s, :] + pos_t[t, :],
 * n = t*S + s, S = (H/p)*(W/p), latent [R, T, H, W, C] f32, patch features in (dh, dw, c)
 * order; all tensors f32.  impl 0: library's choice; 1: the general kernel; 2: the
 * matrix-core kernel (p = 2, C = 16, D a multiple of 256; FC_ERR_UNSUPPORTED otherwise). */
int fc_op_patch_embed(const float* latent, int32_t R, int32_t B, const float* Wp, const float* bp,
                      const float* pos_sp, const float* pos_t, float* x, int32_t T, int32_t H,
                      int32_t W, int32_t C, int32_t p, int32_t D, int32_t rows_per_b,
                      int32_t row_off, int32_t impl, void* hip_stream);

/* Fused guidance + DDIM update on n elements per request, R requests:
 * eps = eps_u + s (eps_c - eps_u) (eps_u NULL: eps = eps_c);
 * x <- c[2] * (x - c[1] eps) / c[0] + c[3] eps, c = fc_schedule_coefficients.
 * eps_out (NULL allowed) receives eps. */
int fc_op_cfg_ddim(float* x, const float* eps_c, const float* eps_u, float* eps_out, size_t n_total,
                   float guidance_scale, const float* coef4_host, void* hip_stream);

/* ---- measurement aid, not part of a step: the rates of a compute unit's matrix pipe and
 * vector pipe under the instruction mix of the attention kernel (bf16 32x32x16 MFMAs, two
 * v_exp_f32 per MFMA), on the part at hand and at the clock it sustains under that load.
 * `blocks` workgroups of 8 waves run `iters` iterations; the first four waves of a workgroup
 * run mode_first, the last four mode_second: 0 idle, 1 four independent MFMA chains per
 * iteration (4 * 32768 FLOP per wave and iteration), 2 eight exponentials per iteration,
 * 3 both interleaved in one instruction stream.  operands: dev, 4096 bf16 (16-byte aligned)
 * that fill the MFMA inputs (random values load the pipe like real data, constants do not);
 * sink: dev, blocks * 512 floats (keeps the work alive); clocks: dev, blocks * 8 pairs of
 * int64: per wave the loop's duration in shader-clock cycles and on the 100 MHz constant
 * counter (their ratio is the sustained shader clock). */
int fc_bench_pipe_rates(const void* operands, int32_t iters, int32_t mode_first, int32_t mode_second,
                        int32_t blocks, float* sink, int64_t* clocks, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FLEXDENOISE_H */
