/*
 * chimera.h - C ABI of one Chimera pipeline worker on one MI355X (gfx950).
 *
 * Chimera (Li & Hoefler, SC'21) runs two pipelines in opposite directions
 * through the same D workers.  Worker i owns stage i of the "down" pipeline
 * and stage D-1-i of the "up" pipeline (section 3.1).  Within one training
 * iteration every worker runs N micro-batches, N/2 through each of its two
 * stages, in the order given by the merged 1F1B schedule; the weight
 * gradients of a stage are summed over its micro-batches with one weight
 * version (section 2, "Convergence friendliness").  This library is that
 * worker: a schedule generator (CPU), a stage (L pre-LayerNorm Transformer
 * blocks, forward and backward, HIP kernels) and the replay of the worker's
 * op list on a HIP stream.  Activations arriving from the previous stage and
 * gradients arriving from the next stage are buffers the caller provides.
 *
 * General rules
 *  - Every function returns CHIMERA_OK (0) or a negative error code; none
 *    aborts or throws.  chimera_last_error() gives the text of the last
 *    failure on the calling thread.
 *  - Pointers named d_* are DEVICE pointers, h_* HOST pointers.  The library
 *    never allocates or frees device memory: the caller owns every device
 *    buffer and must keep it alive while the stage uses it.
 *  - A stage enqueues all its work on the HIP stream given to
 *    chimera_stage_bind (a hipStream_t passed as void*; NULL = default
 *    stream).  Calls return once the work is enqueued unless stated otherwise.
 *  - A stage and the worker binding are not thread-safe.
 *
 * Tensor layouts.  M = microbatch*seq tokens, H = hidden, d = H/heads.
 * Activations are row-major [M, H], token index = b*seq + s.  Element type is
 * the stage dtype (float or bf16); parameter gradients are always float.
 * Parameters live in ONE flat buffer, block after block, inside a block in
 * this order (all row-major, linear maps stored [in, out], y = x W + b):
 *     ln1_g[H] ln1_b[H] w_qkv[H,3H] b_qkv[3H] w_o[H,H] b_o[H]
 *     ln2_g[H] ln2_b[H] w_fc1[H,4H] b_fc1[4H] w_fc2[4H,H] b_fc2[H]
 * w_qkv's columns are [Q | K | V]; head j owns columns j*d..(j+1)*d-1 of each.
 * The gradient buffer has the same order and element counts.
 * One block computes (the paper leaves the block unspecified; this is the
 * GPT-2 style reading):
 *     x1 = x + (Attn(LN1(x) w_qkv + b_qkv)) w_o + b_o
 *     y  = x1 + GeLU(LN2(x1) w_fc1 + b_fc1) w_fc2 + b_fc2
 * LayerNorm: biased variance, eps 1e-5.  Attention: softmax(q k^T / sqrt(d))
 * with an optional causal mask (key <= query).
 */
#ifndef CHIMERA_H
#define CHIMERA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CHIMERA_OK = 0,
    CHIMERA_EINVAL = -1,  /* bad argument                                   */
    CHIMERA_ENOMEM = -2,  /* a caller-provided buffer or capacity too small */
    CHIMERA_ESTATE = -3,  /* call out of order (see each function)          */
    CHIMERA_EDEVICE = -4  /* a HIP call failed                              */
};

enum { CHIMERA_F32 = 0, CHIMERA_BF16 = 1 };

/* schedule algorithms */
enum {
    CHIMERA_DIRECT = 0,   /* Chimera, direct concatenation of basic units (sections 3.1, 3.5) */
    CHIMERA_GPIPE = 1,
    CHIMERA_1F1B = 2,
    CHIMERA_DOUBLING = 3, /* Chimera with forward doubling (section 3.5)                      */
    CHIMERA_HALVING = 4   /* Chimera with backward halving (section 3.5)                      */
};

/* op kinds of a schedule */
enum {
    CHIMERA_OP_F = 0,     /* forward of micro-batch mb                                          */
    CHIMERA_OP_B = 1,     /* backward of micro-batch mb                                         */
    CHIMERA_OP_F2 = 2,    /* forward of micro-batches mb and mb+1 together (mb even)            */
    CHIMERA_OP_BH0 = 3,   /* backward of the first half of micro-batch mb's sequences           */
    CHIMERA_OP_BH1 = 4,   /* backward of the second half                                        */
    CHIMERA_OP_KINDS = 5
};

/* stage options (chimera_stage_set_option) */
enum {
    CHIMERA_OPT_CAUSAL = 0,  /* 1 (default) = causal mask, 0 = bidirectional        */
    CHIMERA_OPT_GELU = 1,    /* 0 (default) = tanh form, 1 = exact erf form         */
    CHIMERA_OPT_KERNELS = 2, /* 0 (default) = matrix-core kernels where the shape   */
                             /* allows, 1 = plain reference kernels everywhere      */
    CHIMERA_OPT_OVERLAP = 3, /* 1 (default) = weight and bias gradients of a        */
                             /* backward run on a second stream of the stage's own, */
                             /* beside the input-gradient chain; 0 = one stream     */
    CHIMERA_OPT_KEEP = 4     /* 1 (default) = a forward keeps its activations for   */
                             /* the backward; 0 = forward-only stage that keeps     */
                             /* nothing (activation recomputation, section 3.5): one */
                             /* scratch slot of at most two blocks, chimera_bwd is   */
                             /* ESTATE, chimera_stage_stash_slot_bytes shrinks       */
};

typedef struct chimera_stage chimera_stage;

/* Text of the last error on this thread; static storage, never NULL. */
const char* chimera_last_error(void);

/* ------------------------------------------------------------------ schedule
 * Section 3.1 (bidirectional 1F1B merge), section 3.5 (direct concatenation
 * of K = N/D basic units) and, as baselines, GPipe and 1F1B-with-flush
 * (section 2, "Bubbles in the pipeline").  Pure CPU; usable without a GPU.
 */
typedef struct {
    int32_t kind;   /* CHIMERA_OP_*: 0 = forward, 1 = backward, ...              */
    int32_t pipe;   /* 0 = down pipeline, 1 = up pipeline (baselines: always 0); */
                    /* with 2f pipelines 2i = down pipeline i, 2i+1 = up pipeline i */
    int32_t mb;     /* global micro-batch id, 0 .. N-1                          */
    int32_t stage;  /* pipeline stage the op belongs to                         */
    int32_t slot;   /* activation-stash slot of that stage used by this         */
                    /* micro-batch (lowest free slot at its forward); -1 for a  */
                    /* doubled forward and the backwards that recompute after it */
    int32_t start;  /* start time when all workers replay as soon as possible   */
                    /* with forward cost = backward cost = 1                    */
    int32_t last_of_stage; /* 1 on the backward that completes this stage's     */
                    /* weight gradients for the iteration (section 3.2)         */
} chimera_op;

/* Op list of worker `rank` in execution order.  Writes min(count, cap) ops to
 * h_out (may be NULL if cap == 0) and the full count (2N) to *h_count.
 * EINVAL: unknown algo; D < 1; N < 1; rank outside [0, D); for CHIMERA_DIRECT
 * also D odd, or N > D and not a multiple of D.  N < D (section 3.1): the micro-batches
 * are split between the two pipelines as evenly as possible, down ids 0..ceil(N/2)-1, up
 * ids ceil(N/2)..N-1; N = 1 runs on the down pipeline alone.
 * ENOMEM: cap < count (list truncated). */
int chimera_schedule(int algo, int D, int N, int rank,
                     chimera_op* h_out, size_t cap, size_t* h_count);

/* Replays all D workers as soon as possible under the data dependencies with
 * integer costs (cost_f, cost_b >= 1).  Outputs (each may be NULL):
 * *h_makespan; h_bubbles[D] = makespan - busy time per worker;
 * h_stash_peak[D] = most micro-batches in flight per worker;
 * h_critical[2] = forwards and backwards on the critical path (section 3.4). */
int chimera_schedule_stats(int algo, int D, int N, int cost_f, int cost_b,
                           int64_t* h_makespan, int64_t* h_bubbles,
                           int32_t* h_stash_peak, int32_t* h_critical);

/* The same for 2f pipelines (section 3.6, Table 3): algo CHIMERA_DIRECT with f down and f up
 * pipelines, f a divisor of D/2 (f = 1 is the call above); other algorithms need f = 1.
 * CHIMERA_DOUBLING needs N = K*D with K >= 2: units of 2D micro-batches, every forward
 * carries two micro-batches (kind F2), every backward one; an odd K leaves one ordinary
 * unit at the end.  CHIMERA_HALVING: the direct order with every backward cut in two
 * halves (kinds BH0, BH1).  Count: 2N ops; 3N for halving; for doubling 3 ops per pair
 * of micro-batches in the doubled units and 2 per micro-batch in an ordinary unit. */
int chimera_schedule_pipes(int algo, int D, int N, int f, int rank,
                           chimera_op* h_out, size_t cap, size_t* h_count);

/* Replay statistics with one integer cost (>= 1) per op kind, h_cost[CHIMERA_OP_KINDS].
 * h_stash_peak_halves[D]: most activations a worker holds, in HALF micro-batches
 * (forward +2, doubled forward +4, backward -2, half backward -1; no recomputation).
 * The paper's figures: Table 3 (bubble ratio (D-2f)/(2fN+D-2f), activations
 * [(D-D/2f+1) M_a, D M_a]); section 3.5 (D-2 bubbles for doubling and halving). */
int chimera_schedule_stats_costs(int algo, int D, int N, int f, const int64_t* h_cost,
                                 int64_t* h_makespan, int64_t* h_bubbles,
                                 int32_t* h_stash_peak_halves, int32_t* h_critical);

/* Worker that holds `stage` of pipeline `pipe` (section 3.1; section 3.6 for f > 1):
 * down pipeline i starts on worker i*(D/f) and walks upwards cyclically, up pipeline i
 * uses the reverse order.  Returns the worker (>= 0) or EINVAL. */
int chimera_pipe_worker(int D, int f, int pipe, int stage);

/* Performance model, Eq. (1) of section 3.4:
 *   T = (F_t + Comm_p2p) C_f + (B_t + Comm_p2p) C_b + max_i Comm_unoverlapped(i),
 * Comm_p2p = alpha + beta*act_words, Comm_allreduce = 2 log2(r) alpha + 2 (r-1) beta
 * grad_words / r with r = 2 f W stage replicas for Chimera and W for GPipe / 1F1B.
 * C_f, C_b come from the as-soon-as-possible replay of the schedule with those op costs.
 * Free regions are a worker's idle intervals: the allreduce of a stage uses the idle time
 * after the stage's last backward (eager != 0) or after the worker's last op (eager == 0),
 * a worker's allreduces run one after the other, and what is left at the end of the
 * computation is unoverlapped.  f_t, b_t in seconds (any unit, consistently), alpha in the
 * same unit, beta in that unit per word.  h_out[7] = {T, F_t C_f + B_t C_b, (C_f + C_b)
 * Comm_p2p, Comm_allreduce, max_i Comm_unoverlapped(i), C_f, C_b}.  Pure CPU. */
int chimera_model_iteration_time(int algo, int D, int N, int f, int W, double f_t, double b_t,
                                 double alpha, double beta, double act_words, double grad_words,
                                 int eager, double* h_out);

/* Configuration selection of section 3.4 (and section 4.3): a candidate is one (W, D, B) with
 * what was measured or computed for it; P = W*D workers train a mini-batch of `minibatch`
 * samples, so a worker runs N = minibatch / (W*B) micro-batches through its pipeline. */
typedef struct {
    int32_t D, W, B;        /* pipeline stages, replicated pipelines, micro-batch size            */
    int32_t recompute;      /* activation recomputation: a backward modelled as 3 F_t, not 2 F_t   */
    double f_t;             /* forward time of one stage at this B (section 3.4: measured)          */
    double b_t;             /* backward time; <= 0: modelled from f_t                                */
    double act_words;       /* one stage-boundary message                                            */
    double grad_words;      /* gradients of one stage                                                */
    double weight_bytes;    /* M_theta: what one stage replica keeps resident on a worker            */
    double act_bytes;       /* M_a: activations of one stage for one micro-batch in flight           */
} chimera_candidate;
typedef struct {
    int32_t valid;          /* 0: W*B does not divide the mini-batch, or the schedule does not exist */
    int32_t N;              /* micro-batches per worker and iteration                                 */
    int32_t fits;           /* mem_bytes <= capacity                                                  */
    int32_t chosen;         /* the largest fitting B of its (W, D): only these compete                */
    int32_t c_f, c_b;       /* critical path                                                          */
    double mem_bytes;       /* worst worker: replicas * M_theta + (most micro-batches held) * M_a     */
    double T;               /* Eq. (1)                                                                */
    double throughput;      /* minibatch / T                                                          */
} chimera_candidate_eval;
/* Evaluates every candidate (memory as in section 3.1 / Table 2: 2f stage replicas per worker for
 * CHIMERA_DIRECT, one otherwise, plus the activations held at the worst moment of the schedule;
 * time by Eq. (1) as chimera_model_iteration_time does), keeps per (W, D) the largest B that
 * fits `capacity_bytes` (the greedy rule of section 3.4), and returns in *h_best the index of
 * the kept candidate with the highest throughput (the first of equals), -1 if none fits.
 * h_eval[count] receives all evaluations.  EINVAL: count < 1, NULL arrays, a non-positive f_t,
 * negative sizes or parameters, algo CHIMERA_DOUBLING / CHIMERA_HALVING.  Pure CPU. */
int chimera_model_select(int algo, int f, int64_t minibatch, double capacity_bytes, double alpha, double beta,
                         int eager, int count, const chimera_candidate* h_cand,
                         chimera_candidate_eval* h_eval, int* h_best);

/* --------------------------------------------------------------------- stage
 * A stage = `layers` Transformer blocks at fixed shape (the paper's F_t / B_t
 * black box, section 3.4).  Returns NULL on error (EINVAL: non-positive size,
 * hidden % heads != 0, hidden % 8 != 0, unknown dtype). */
chimera_stage* chimera_stage_create(int layers, int hidden, int heads, int seq,
                                    int microbatch, int dtype);
/* Only before chimera_stage_bind; ESTATE afterwards. */
int chimera_stage_set_option(chimera_stage* st, int key, int value);
void chimera_stage_destroy(chimera_stage* st);

/* Sizes in bytes of the buffers the caller must provide. */
size_t chimera_stage_weight_bytes(const chimera_stage* st);
size_t chimera_stage_grad_bytes(const chimera_stage* st);
size_t chimera_stage_stash_slot_bytes(const chimera_stage* st);
size_t chimera_stage_workspace_bytes(const chimera_stage* st);

/* Hands the stage its device buffers (all 256-byte aligned): weights
 * (weight_bytes, stage dtype), gradients (grad_bytes, float), the activation
 * stash (stash_slots * stash_slot_bytes), scratch (workspace_bytes) and the
 * stream.  The stash holds what the backward of an in-flight micro-batch needs
 * (the paper's M_a per slot; Chimera needs between D/2+1 and D slots per
 * worker over its two stages, Table 2).  Buffers are borrowed, not copied. */
int chimera_stage_bind(chimera_stage* st, const void* d_weights, float* d_grads,
                       void* d_stash, int stash_slots, void* d_workspace,
                       void* hip_stream);

/* Registers the buffers of micro-batch `mb` (any non-negative id): d_x_in
 * [M,H] activation from the previous stage, d_y_out [M,H] activation for the
 * next stage, d_dy_in [M,H] gradient from the next stage, d_dx_out [M,H]
 * gradient for the previous stage.  d_x_in is read again by the backward, so
 * it must stay unchanged until chimera_bwd(mb) has run. */
int chimera_stage_set_io(chimera_stage* st, int mb, const void* d_x_in, void* d_y_out,
                         const void* d_dy_in, void* d_dx_out);

/* Forward of micro-batch mb: takes a free stash slot (or `slot` >= 0 via
 * chimera_fwd_slot), writes d_y_out.  ESTATE: stage not bound, io of mb not
 * set, mb already in flight, no free slot / slot taken. */
int chimera_fwd(chimera_stage* st, int mb);
int chimera_fwd_slot(chimera_stage* st, int mb, int slot);
/* Backward of micro-batch mb: writes d_dx_out, ADDS this micro-batch's
 * parameter gradients to d_grads (float accumulation in call order), frees
 * the slot.  ESTATE: forward of mb not done. */
int chimera_bwd(chimera_stage* st, int mb);
/* Backward halving (section 3.5): the backward of micro-batch mb in two parts, half 0 =
 * its first microbatch/2 sequences, half 1 = the rest, each a backward at half the
 * micro-batch size over the same stash slot; the two calls together add exactly the
 * gradients chimera_bwd(mb) would add and write the same dx.  Half 0 must come first;
 * half 1 frees the slot.  EINVAL if microbatch is odd; ESTATE when out of order. */
int chimera_bwd_half(chimera_stage* st, int mb, int half);

int chimera_stage_in_flight(const chimera_stage* st);
/* Starts a new iteration: the stage's gradients count as zero from now on.  The zeroing
 * itself is deferred - the next backward WRITES every gradient instead of accumulating
 * (no fill pass and no read of the old values; one weight version per iteration, section 2),
 * or, where a kernel on the path cannot overwrite, fills the buffer first.  The contents of
 * d_grads are therefore unspecified between this call and the next chimera_bwd /
 * chimera_bwd_half / chimera_stage_read_grads (which zero-fills if nothing ran); a caller
 * that reads d_grads itself does so after the backwards of the iteration. */
int chimera_stage_zero_grads(chimera_stage* st);
/* Copies the gradient buffer to host memory and waits for the stream. */
int chimera_stage_read_grads(chimera_stage* st, float* h_dst, size_t bytes);

/* -------------------------------------------------------------------- worker
 * Section 3.1: a worker = its down stage and its up stage.  Both must be bound
 * and have the io of every micro-batch they will see registered:
 * the down stage sees ids k*D + 0..D/2-1, the up stage ids k*D + D/2..D-1. */
int chimera_worker_bind(chimera_stage* down_stage, chimera_stage* up_stage);
/* Replays chimera_schedule(CHIMERA_DIRECT, D, N, rank) on the bound stages in
 * list order, using each op's stash slot, and waits for the stream(s) once at
 * the end.  ENOMEM if a stage was bound with fewer slots than the schedule
 * needs.  Both stages must have no micro-batch in flight. */
int chimera_run_worker(int rank, int D, int N);
/* Same for any algorithm; for the one-pipeline baselines only the down stage
 * is used and holds stage `rank`. */
int chimera_run_worker_algo(int algo, int rank, int D, int N);
/* 2f pipelines (section 3.6): h_stages[p] is the stage of pipeline p (2i = down pipeline i,
 * 2i+1 = up pipeline i) that this worker holds, count = 2f.  chimera_worker_bind(d, u) is
 * the same with count 2.  Unbinds any doubled stages. */
int chimera_worker_bind_pipes(chimera_stage* const* h_stages, int count);
/* Forward doubling (section 3.5): besides the worker's two stages, two forward-only stages
 * (CHIMERA_OPT_KEEP = 0) of the same shape at TWICE the micro-batch, bound to the same
 * weight buffers.  The io of double micro-batch (g, g+1), g even, is registered on them under
 * id g: x and y are [2*microbatch, seq, H] (dy, dx are not used and may repeat x, y).
 * EINVAL when shapes or weights do not match; ESTATE without a bound worker. */
int chimera_worker_bind_doubling(chimera_stage* down2, chimera_stage* up2);
/* Replays chimera_schedule_pipes(algo, D, N, f, rank).  Op kinds: F forward into the op's
 * stash slot; B backward - if the micro-batch's activations were not kept (it went through a
 * doubled forward) the forward is run again first into a free slot (activation
 * recomputation); F2 forward of two micro-batches on the doubled stage; BH0/BH1 the two
 * halves of a backward.  With doubling every stage needs one stash slot more than the
 * largest slot index in its ops.  One wait per stream at the end. */
int chimera_run_worker_pipes(int algo, int rank, int D, int N, int f);
/* on != 0: bracket every op of the next replays with HIP events (off by default). */
int chimera_worker_set_timing(int on);
/* Milliseconds the last chimera_run_worker* spent in forward ops and in
 * backward ops (HIP events around every op), and the op counts. */
int chimera_worker_last_timing(double* h_fwd_ms, double* h_bwd_ms, int* h_nf, int* h_nb);
/* Host milliseconds the last chimera_run_worker* needed to build the schedule and enqueue
 * every launch, i.e. up to (not including) its wait for the streams: the replay is bound by
 * the host once this approaches the iteration time. */
int chimera_worker_last_enqueue_ms(double* h_ms);

/* Per-kernel-class timing of everything the stages launch while enabled: a HIP
 * event pair brackets every launch (this slows the replay a little, so keep it
 * off when timing whole iterations).  Classes: 0 GEMM forward, 1 GEMM dgrad,
 * 2 GEMM wgrad, 3 attention forward, 4 attention backward, 5 LayerNorm forward,
 * 6 LayerNorm backward, 7 column sums, 8 the second launch of a block's weight
 * gradients (row bands that leave the 256x256 launch for smaller tiles; class 2 is
 * then the first launch alone).  chimera_profile_read must be called
 * with the stream idle; it returns the summed milliseconds, the number of
 * launches and the summed algorithmic work (flop for classes 0-4 and 8, bytes for
 * 5-7) since the last chimera_profile_reset. */
int chimera_profile_enable(int on);
int chimera_profile_reset(void);
int chimera_profile_read(int cls, double* h_ms, long long* h_launches, double* h_work);

/* ---------------------------------------------------------- single operators
 * The kernels a stage is made of, callable on raw device buffers so that each
 * can be checked and profiled alone.  dtype as above; `impl` 0 = the kernel
 * the stage would pick, 1 = plain reference kernel.  All enqueue on
 * `hip_stream`.
 *
 * GEMM  C[m,n] = sum_k A(i,k) B(k,j) with epilogue.  a_kc != 0: A stored
 * [m, k] (k contiguous, leading dimension lda); a_kc == 0: A stored [k, m].
 * b_kc != 0: B stored [n, k] (k contiguous); b_kc == 0: B stored [k, n].
 * epilogue: 0 C = acc (dtype); 1 C = acc + bias[n]; 2 C = acc + bias[n] and
 * C2 = GeLU(C); 3 C = acc + bias[n] + R[m,n]; 4 C = acc * GeLU'(R[m,n]);
 * 5 C (float, always) += acc.  C, C2, R have leading dimension n.
 * EINVAL if k, n or a leading dimension is not a multiple of 8.
 * d_workspace (may be NULL): chimera_op_gemm_workspace_bytes(m, n, k) bytes, 256-byte
 * aligned, whose first 4096 bytes are zero before the first call; with it, and with a
 * forced tile of 256x256 and splits > 1 (chimera_op_gemm_tuning), the bf16
 * kernel splits the k range over several workgroups per tile (partial sums are added in
 * a fixed order, so results stay reproducible).  Concurrent calls need separate
 * workspaces.  Without it every product runs unsplit. */
size_t chimera_op_gemm_workspace_bytes(int m, int n, int k);
/* Tuning aid for the bf16 matrix-core products (process-wide, affects later launches
 * of every stage; not thread-safe against running launches).  tile_m x tile_n: 0x0 =
 * chosen per shape (default), 128x128 or 256x256 forced; splits: 0/1 = none, 2..8 =
 * split-K with a 256x256 forced tile and a workspace; async_mode: 0 = automatic,
 * 1 = register-staged kernels, 2 = k-sliced 8-wavefront form for every 128x128 launch,
 * 3 = never that form.  The initial state comes from the environment variables
 * CHIMERA_GEMM_TILE ("256x256", "256x256x4") and CHIMERA_GEMM_ASYNC ("0", "4k", other),
 * read once at first use.  EINVAL for any other value. */
int chimera_op_gemm_tuning(int tile_m, int tile_n, int splits, int async_mode);
/* For reports: the kernel instantiation(s) the calling thread's last grouped launch
 * (chimera_op_gemm_group_accumulate, or a block's weight gradients inside chimera_bwd) went
 * to, e.g. "gemm_bf16_async_group_kernel<256,256,2,4,1,2,false,false>"; two names joined by
 * " + " when the last row bands went out as a second launch.  Thread-local static storage,
 * never freed by the caller; "" before the first such launch. */
const char* chimera_op_gemm_group_last_kernel(void);
int chimera_op_gemm(int dtype, int impl, int epilogue, int gelu_kind,
                    int m, int n, int k,
                    const void* d_a, int lda, int a_kc,
                    const void* d_b, int ldb, int b_kc,
                    const void* d_bias, const void* d_r,
                    void* d_c, void* d_c2, void* d_workspace, size_t workspace_bytes,
                    void* hip_stream);
/* `count` (1..4) products C_p[m_p, n_p] (float) += A_p^T-stored-[k, m_p] x B_p-stored-[k, n_p]
 * in ONE launch: the weight gradients dW += X^T dY of one Transformer block (gradient
 * accumulation over micro-batches, section 3.1 of the paper; the four linear layers of a
 * block, section 4.1).  bf16 operands only, one contraction length k (a multiple of 64) for
 * all products, m_p and n_p multiples of 8 and at least 8, 16-byte aligned pointers,
 * leading dimensions lda_p >= m_p, ldb_p >= n_p (multiples of 8), C_p has leading dimension
 * n_p.  h_bsum (may be NULL, and so may any entry): bsum_p[j] (float, n_p entries) +=
 * sum over k of B_p(k, j), the bias gradient that belongs to dW_p; it costs no extra pass
 * over B.  The h_* arguments are host arrays of `count` entries (read before the call
 * returns); the pointers in them are device pointers.  The C_p equal `count` calls of
 * chimera_op_gemm with epilogue 5.  overwrite != 0: C_p and bsum_p RECEIVE the products and
 * sums (their old contents are neither read nor kept) - the first micro-batch of an
 * iteration.  EINVAL for anything else (nothing is launched). */
int chimera_op_gemm_group_accumulate(int count, const int* h_m, const int* h_n, int k,
                                     const void* const* h_a, const int* h_lda,
                                     const void* const* h_b, const int* h_ldb,
                                     float* const* h_c, float* const* h_bsum, int overwrite,
                                     void* hip_stream);
/* y = LN(x) gamma + beta; mean, rstd [rows] float are written for the backward. */
int chimera_op_layernorm_fwd(int dtype, int rows, int cols, const void* d_x,
                             const void* d_gamma, const void* d_beta, void* d_y,
                             float* d_mean, float* d_rstd, void* hip_stream);
/* dx = res + LN'(dy); dgamma, dbeta (float) += column sums.  d_scratch: float
 * [layernorm_bwd_scratch_floats(rows, cols)]. */
size_t chimera_op_layernorm_bwd_scratch_floats(int rows, int cols);
int chimera_op_layernorm_bwd(int dtype, int rows, int cols, const void* d_dy,
                             const void* d_x, const float* d_mean, const float* d_rstd,
                             const void* d_gamma, const void* d_res, void* d_dx,
                             float* d_dgamma, float* d_dbeta, float* d_scratch,
                             void* hip_stream);
/* chimera_op_layernorm_bwd for callers that cannot allocate device memory or pass a
 * workspace (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): same kernels and same results, but the per-block partial sums of dgamma and
 * dbeta live in an array of the library's own, a file-scope device array of
 * chimera_op_layernorm_bwd_noalloc_max_scratch_floats() floats (16 MiB) that every GPU the
 * library runs on holds until the process ends.  Inputs and outputs are the caller's device
 * buffers as above.  The call allocates nothing (no hipMalloc / hipFree, no allocating
 * library routine); the array's device address is looked up once per device, on the first
 * call with that device current.  ENOMEM, with nothing launched, when
 * chimera_op_layernorm_bwd_scratch_floats(rows, cols) exceeds the array (e.g. 4096 x 2048
 * bf16 still fits, 8192 x 2048 does not).  Every call on a GPU shares that GPU's array and its
 * kernels overwrite the part they read, so nothing has to be cleared between calls - but
 * calls that overlap on one GPU (different streams, or threads) race on it: serialise them. */
size_t chimera_op_layernorm_bwd_noalloc_max_scratch_floats(void);
int chimera_op_layernorm_bwd_noalloc(int dtype, int rows, int cols, const void* d_dy,
                                     const void* d_x, const float* d_mean, const float* d_rstd,
                                     const void* d_gamma, const void* d_res, void* d_dx,
                                     float* d_dgamma, float* d_dbeta, void* hip_stream);
/* out[cols] (float) += sum over rows of x[rows, cols]. */
size_t chimera_op_colsum_scratch_floats(int rows, int cols);
int chimera_op_colsum(int dtype, int rows, int cols, const void* d_x, float* d_out,
                      float* d_scratch, void* hip_stream);
/* ctx[M,H] = softmax(q k^T / sqrt(d) [+ causal mask]) v per (sequence, head),
 * q, k, v read from qkv [M, 3H]; lse [batch, heads, seq] float = log-sum-exp
 * of the scaled scores (kept for the backward). */
int chimera_op_attention_fwd(int dtype, int impl, int batch, int seq, int heads, int head_dim,
                             int causal, const void* d_qkv, void* d_ctx, float* d_lse,
                             void* hip_stream);
/* dqkv [M,3H] from dctx [M,H]; d_delta: float scratch [batch*heads*seq]. */
int chimera_op_attention_bwd(int dtype, int impl, int batch, int seq, int heads, int head_dim,
                             int causal, const void* d_qkv, const void* d_ctx,
                             const float* d_lse, const void* d_dctx, void* d_dqkv,
                             float* d_delta, void* hip_stream);

/* ------------------------------------------------------- the pipeline's two ends
 * Section 4.1 of the paper: the first stage of a language model carries an extra embedding
 * layer; the last stage ends in the loss.  GPT-2 reading (token + learned position table;
 * final LayerNorm, untied vocabulary projection, cross-entropy).  All sums have a fixed order
 * (no atomics).  Token and target ids must lie in [0, vocab); ids outside are clamped into the
 * table (never followed out of bounds).  hidden must be a multiple of 8, and so must vocab
 * wherever it is a matrix dimension (cross-entropy, head).
 *
 * x[t] = wte[token[t]] + wpe[t mod seq];  wte [vocab, hidden], wpe [seq, hidden], x [tokens, hidden]
 * in the given dtype; d_tokens int32 [tokens], tokens a multiple of seq. */
int chimera_op_embedding_fwd(int dtype, int tokens, int seq, int hidden, int vocab,
                             const int32_t* d_tokens, const void* d_wte, const void* d_wpe,
                             void* d_x, void* hip_stream);
/* dwte[v] += sum of dx[t] over the positions t with token[t] = v (ascending t),
 * dwpe[p] += sum of dx[b*seq + p] over the sequences b (ascending); both float. */
int chimera_op_embedding_bwd(int dtype, int tokens, int seq, int hidden, int vocab,
                             const int32_t* d_tokens, const void* d_dx,
                             float* d_dwte, float* d_dwpe, void* hip_stream);
/* In place over d_logits [rows, vocab]: z <- scale * (softmax(z) - onehot(target)) row by row,
 * d_loss_rows[t] = scale * (logsumexp(z[t]) - z[t, target[t]]) and d_loss[0] += their sum. */
int chimera_op_softmax_xent(int dtype, int rows, int vocab, void* d_logits, const int32_t* d_targets,
                            float scale, float* d_loss_rows, float* d_loss, void* hip_stream);
/* The last stage's head, forward and backward in one call (at the last stage the backward
 * follows its forward immediately, section 3.1):
 *   h = LayerNorm(y; lnf_g, lnf_b),  z = h W_head (W_head stored [hidden, vocab]),
 *   d_loss[0] += scale * sum_t (logsumexp(z[t]) - z[t, target[t]]),
 *   d_dy = dLoss/dy [tokens, hidden] (dtype),  d_dlnf_g, d_dlnf_b [hidden], d_dw_head
 *   [hidden, vocab] (float) += their gradients.
 * `scale` is the weight of these tokens in the mini-batch loss (1 / token count for a mean).
 * d_workspace: chimera_head_workspace_bytes(dtype, tokens, hidden, vocab) bytes, 256-byte
 * aligned (it holds h, the logits and their gradient).  ENOMEM if it is too small. */
size_t chimera_head_workspace_bytes(int dtype, int tokens, int hidden, int vocab);
int chimera_head_loss(int dtype, int tokens, int hidden, int vocab, const void* d_y,
                      const int32_t* d_targets, const void* d_lnf_g, const void* d_lnf_b,
                      const void* d_w_head, float scale, void* d_dy, float* d_dlnf_g,
                      float* d_dlnf_b, float* d_dw_head, float* d_loss, void* d_workspace,
                      size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------ measured ceilings
 * What the device sustains, to set beside the published peaks when the stage kernels'
 * rates are reported (measurement only; the hot path never calls them).
 * chimera_probe_mfma_bf16: every SIMD of the chip runs `iters` x 16 bf16 32x32x16 MFMAs on
 * register-resident operands; *h_tflops receives the rate.  d_sink: 4 bytes of device
 * memory (never written).  chimera_probe_copy: dst = src over `bytes` bytes (a multiple of
 * 16, both pointers 16-byte aligned, buffers owned by the caller); *h_gbs receives
 * (bytes read + bytes written) per second.  Both wait for their own launches. */
int chimera_probe_mfma_bf16(float* d_sink, int iters, double* h_tflops, void* hip_stream);
int chimera_probe_copy(const void* d_src, void* d_dst, size_t bytes, double* h_gbs, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CHIMERA_H */
