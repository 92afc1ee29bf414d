/*
 * libga -- the parameter-server master of Gap-Aware asynchronous SGD on one
 * AMD MI355X (gfx950).
 *
 * Paper: Barkai, Hakimi, Schuster, "Gap-Aware Mitigation of Gradient
 * Staleness", ICLR 2020.  Notation: the paper writes d for the number of
 * parameters and N for the number of workers; this header writes N for the
 * number of parameters and n_workers (W) for the number of workers.
 *
 * A context is one master (App. C.1: the master is a FIFO over worker
 * arrivals).  It owns, inside a caller-provided device workspace:
 *   theta[N]            master parameters                     (Sec. 2)
 *   v[N]                update (momentum) vector              (Sec. 2, Alg. 2)
 *   m[N]                biased second moment of v             (Alg. 14)
 *   snap[W][N]          theta^i, what was last sent to worker i (Alg. 4: "save
 *                       and send"; App. C.1: theta^i = theta_{k - tau_k})
 * and on the host: the step counter k and iter[W] (Alg. 3 / Alg. 5).
 * All state is float.  Gradients are float or bfloat16.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses.  The library never allocates or frees device memory: every
 *     device buffer, including the workspace, belongs to the caller and must
 *     stay valid until ga_destroy.  The library owns only the host-side ga_ctx
 *     (with a few hundred KB of pinned host memory for staging the arrival table).
 *   - Every call that touches the device enqueues on the HIP stream given to
 *     ga_create and returns without waiting, unless stated otherwise.
 *   - Every function returning int returns a ga_status; ga_last_error(ctx)
 *     describes the failure.  No exception crosses this boundary.  Arguments
 *     are checked before anything is enqueued: after GA_ERR_ARG,
 *     GA_ERR_WORKER, GA_ERR_ALIGN or GA_ERR_STATE nothing has been enqueued
 *     and no state has changed.  GA_ERR_HIP (a HIP runtime call failed) can
 *     come in the middle of a call that enqueues several operations: what was
 *     enqueued before it stays enqueued, the host bookkeeping covers exactly
 *     the arrivals whose launch succeeded (ga_step tells how many), and a
 *     failed ga_create_ex may have enqueued the fill of the workspace.
 *   - A context is not thread safe: one master, one caller at a time.
 *
 * Arithmetic of one arrival (worker i, gradient g, master step k >= 1,
 * tau_k = k - iter[i]), per parameter j, every line one IEEE float operation:
 *   GA modes (Alg. 4, Eq. 5; C from Alg. 14 as left by arrival k-1):
 *       diff  = theta - snap_i            delta = |diff|
 *       mhat  = m * inv_bc_prev           inv_bc_prev = 1/(1 - beta^(k-1)), 0 when k = 1
 *       C     = eta_max * (sqrt(mhat) + eps)
 *       Graw  = delta / C
 *       G     = 1 + Graw   (GA_MODE_GA)   or   max(1, Graw)   (GA_MODE_GA_HINGE)
 *       ghat  = g / G
 *   GA_MODE_SA (Alg. 5):      ghat = g / tau_k
 *   otherwise:                ghat = g
 *   v     = gamma * v + ghat                                   (Alg. 2 / 4 / 5)
 *   theta = theta - lr * v,   lr = eta_k, or eta_k / tau_k for GA_MODE_SA_STEP (Alg. 3)
 *   m     = beta * m + (1 - beta) * (v * v)                    (Alg. 14; GA modes, or gap tracking on)
 *   snap_i = theta                                             (Alg. 4)
 * then on the host iter[i] = k.  The scalar 1/(1 - beta^(k-1)) is evaluated in
 * double and rounded once to float (Alg. 14 divides by 1 - beta^k and leaves
 * the rounding open; before the first arrival m-hat_0 = 0).
 *
 * Two choices above are readings that nothing in the paper pins: Alg. 14 is
 * fed with the update vector v actually taken (it prints v <- gamma v + g with
 * the raw gradient, while Alg. 4 keeps g / G in v; one v is kept here), and
 * GA_MODE_GA_HINGE is a variant of this library, not the paper's penalty.
 */
#ifndef GA_H
#define GA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ga_ctx ga_ctx;

enum ga_mode {
    GA_MODE_ASGD = 0,     /* Alg. 2: no penalty */
    GA_MODE_SA = 1,       /* Alg. 5: gradient divided by the delay */
    GA_MODE_SA_STEP = 2,  /* Alg. 3: step size divided by the delay */
    GA_MODE_GA = 3,       /* Alg. 4: gradient divided by G = |diff|/C + 1 */
    GA_MODE_GA_HINGE = 4  /* variant: gradient divided by max(1, |diff|/C) */
};

/* Which master algorithm family the context runs.  The penalty mode applies
 * inside each family:
 *   MOMENTUM: Alg. 2 (ASGD), Alg. 5 (SA), Alg. 3 (SA_STEP), Alg. 4 (GA, GA_HINGE)
 *   DANA:     Alg. 6 (ASGD), Alg. 7 (SA), Alg. 8 (GA, GA_HINGE)
 *   ADAM:     Alg. 9 (ASGD), Alg. 10 (SA), Alg. 11 (GA, GA_HINGE)
 * GA_MODE_SA_STEP exists for MOMENTUM only.
 *
 * DANA, per parameter (v_i = momentum of the arriving worker, vsum = sum_j v_j):
 *   ghat = g / G (GA modes, G as in the header comment) | g / tau (SA) | g
 *   vnew = gamma * v_i + ghat ;  theta = theta - eta_k * vnew
 *   vsum = (vsum - v_i) + vnew ;  v_i = vnew
 *   m    = beta * m + (1 - beta) * (vnew * vnew)             (Alg. 14 on the step taken)
 *   snap_i = theta - (eta_k * gamma) * vsum                   (look-ahead estimate sent to the worker)
 * ADAM, per parameter (m1, v2 = Adam moments; m = Alg. 14 state of the update vector u):
 *   coef = (1 - beta1) / G (GA modes) | (1 - beta1) / tau (SA) | (1 - beta1)
 *   m1 = beta1 * m1 + coef * g ;  v2 = beta2 * v2 + (1 - beta2) * (g * g)
 *   u  = (m1 * ib1) / (sqrt(v2 * ib2) + adam_eps),  ib = (float)(1 / (1 - beta^k)) in double
 *   theta = theta - eta_k * u ;  m = beta * m + (1 - beta) * (u * u) ;  snap_i = theta
 */
enum ga_family { GA_FAMILY_MOMENTUM = 0, GA_FAMILY_DANA = 1, GA_FAMILY_ADAM = 2 };

enum ga_dtype { GA_F32 = 0, GA_BF16 = 1 };

/* Device arrays of a context, for ga_get_array / ga_put_array. */
enum ga_array {
    GA_ARR_THETA = 0,
    GA_ARR_V = 1,         /* MOMENTUM: v;  DANA: vsum;  ADAM: m1 */
    GA_ARR_M = 2,         /* Alg. 14 state */
    GA_ARR_SNAPSHOT = 3,  /* per worker */
    GA_ARR_WORKER_V = 4,  /* DANA only, per worker: v_i */
    GA_ARR_ADAM_V2 = 5    /* ADAM only */
};

enum ga_status {
    GA_OK = 0,
    GA_ERR_ARG = -1,     /* null pointer, zero size, value out of range, unknown enum */
    GA_ERR_WORKER = -2,  /* worker id >= n_workers */
    GA_ERR_ALIGN = -3,   /* workspace not 256-byte aligned or too small */
    GA_ERR_STATE = -4,   /* call not valid in the context's current state */
    GA_ERR_HIP = -5      /* a HIP runtime call failed */
};

/* Iteration-time models of the arrival-schedule simulator. */
enum ga_time_dist {
    GA_DIST_EXP = 0,          /* Exp(mean 1) per iteration */
    GA_DIST_LOGNORMAL = 1,    /* exp(sigma z) per iteration, z ~ N(0,1) */
    GA_DIST_HETERO = 2,       /* worker mean exp(sigma z_w), times Exp(1) per iteration */
    GA_DIST_GAMMA_HOMO = 3,   /* Alg. 12: q = G(a_task, mean/a_task) once; time = G(a_mach, q/a_mach) */
    GA_DIST_GAMMA_HETERO = 4  /* Alg. 13: p[w] = G(a_mach, mean/a_mach) per worker; time = G(a_task, p[w]/a_task) */
};

/* Time model for ga_simulate_schedule_ex / ga_simulate_speedup.  The gamma
 * model is the one of App. C.3: a_task = 1/v_task^2, a_mach = 1/v_mach^2,
 * mu_task = mu_mach = mean; the paper uses v_task = 0.1 and v_mach = 0.1
 * (homogeneous) or 0.6 (heterogeneous).  G(alpha, scale) with alpha >= 1 is
 * drawn with the Marsaglia-Tsang method from counter-based uniforms. */
typedef struct ga_time_model {
    int dist;       /* ga_time_dist */
    double sigma;   /* LOGNORMAL, HETERO */
    double mean;    /* GAMMA_*: > 0 */
    double v_mach;  /* GAMMA_*: in (0, 1] */
    double v_task;  /* GAMMA_*: in (0, 1] */
} ga_time_model;

enum ga_source_kind { GA_SRC_QUADRATIC_NOISE = 0, GA_SRC_BUFFERS = 1 };
enum ga_pick { GA_PICK_BY_WORKER = 0, GA_PICK_BY_ARRIVAL = 1 };

/*
 * Where ga_run_schedule takes the gradient of each arrival from.  The source
 * stands in for the workers of Alg. 1.
 *
 * GA_SRC_QUADRATIC_NOISE: the worker holds theta_w = snap_i and returns, per
 *   parameter j at master step k,
 *       g = a[j] * (theta_w[j] - theta_star[j]) + sigma * z(seed, k, j)
 *   with z the counter-based standard normal documented at ga_noise_fill.
 *   dev_a and dev_theta_star are device arrays of N floats, 16-byte aligned.
 *   persistent != 0 (parameter-wise Gap only): all arrivals are replayed inside
 *   one kernel per chunk of the schedule (no per-arrival launch); persistent == 0: one gradient launch
 *   and one update launch per arrival, through dev_scratch_g (N floats,
 *   16-byte aligned device buffer, required in that case only).
 *
 * GA_SRC_BUFFERS: precomputed gradients.  host_dev_bufs is a HOST array of
 *   n_bufs DEVICE pointers, each to N values of `dtype`.  Arrival k of worker i
 *   uses buffer (i mod n_bufs) for GA_PICK_BY_WORKER, ((k-1) mod n_bufs) for
 *   GA_PICK_BY_ARRIVAL.  persistent == 0: one update launch per arrival.
 *   persistent != 0 (parameter-wise Gap only; every buffer aligned to four
 *   values: 16 bytes for GA_F32, 8 for GA_BF16, else GA_ERR_ALIGN): the
 *   arrivals of the call are a queue whose gradients are all present, and
 *   each chunk of up to 8192 of them is applied by one launch that keeps
 *   theta, v and m in registers and touches only the gradient and the
 *   snapshot of each arrival.  The arrivals are applied in schedule order
 *   with the arithmetic of the per-arrival kernel: the results are the same
 *   bits.  The buffers must not change before the stream has finished.
 */
typedef struct ga_grad_source {
    int kind; /* ga_source_kind */
    /* GA_SRC_QUADRATIC_NOISE */
    const float* dev_a;
    const float* dev_theta_star;
    uint64_t seed;
    float sigma;
    int persistent;
    float* dev_scratch_g;
    /* GA_SRC_BUFFERS */
    const void* const* host_dev_bufs;
    uint32_t n_bufs;
    int dtype; /* ga_dtype */
    int pick;  /* ga_pick */
} ga_grad_source;

/* Gap statistics of one worker against the current master state (App. C.8
 * plots the average Gap).  Graw = |theta - snap_i| / C; the paper's Gap is
 * Graw + 1.  Non-finite Graw values are counted and left out of the mean. */
typedef struct ga_diag {
    double mean_graw;      /* sum of finite Graw / N */
    double frac_gt1;       /* #{Graw > 1} / N: parameters the hinge form penalises */
    double frac_gt0;       /* #{Graw > 0} / N: parameters the paper's form penalises */
    uint64_t n_nonfinite;  /* #{Graw is inf or nan} */
} ga_diag;

/* One row of the per-arrival table that the host bookkeeping produces and the
 * kernels consume (Alg. 3 / Alg. 5 bookkeeping; Alg. 14 bias correction). */
typedef struct ga_arrival {
    uint32_t worker;  /* i */
    float tau;        /* (float) tau_k */
    float lr;         /* eta_k, or eta_k / tau_k for GA_MODE_SA_STEP */
    float inv_bc_prev; /* (float)(1 / (1 - beta^(k-1))); 0 when k = 1 */
} ga_arrival;

/* How many parameters share one Gap (Sec. 4.3).  PARAMETER is Eq. 5 (the
 * paper's choice).  LAYER is Eq. 4: per layer p,
 *     G_p = ||theta_p - snap_i,p|| / C_p + 1,   C_p = eta_max * (sqrt(sum_{j in p} mhat_j) + eps)
 * (hinge mode: max(1, ||.|| / C_p)), and every gradient element of the layer is
 * divided by G_p.  GLOBAL is Def. 1: one layer holding all parameters.  The
 * two sums are accumulated in double and rounded once to float.  LAYER and
 * GLOBAL exist for the MOMENTUM family in the two GA modes, one arrival per
 * launch sequence (reduce, per-layer Gap, update); not in the persistent kernel,
 * which would need a grid-wide reduction per arrival. */
enum ga_gap_scope { GA_GAP_PARAMETER = 0, GA_GAP_LAYER = 1, GA_GAP_GLOBAL = 2 };

/* Full configuration of a master, for ga_create_ex.  Fill with ga_config_init
 * first, then change what differs. */
typedef struct ga_config {
    uint64_t N;
    uint32_t n_workers;
    int family;      /* ga_family, default GA_FAMILY_MOMENTUM */
    int mode;        /* ga_mode, default GA_MODE_GA */
    float eta;       /* eta_k = eta_max, default 0.1 */
    float gamma;     /* momentum coefficient, |gamma| < 1, default 0.9; ignored by ADAM */
    float beta;      /* Alg. 14 decay, default 0.999 */
    float eps;       /* Alg. 14 epsilon, default 1e-8 */
    float adam_beta1, adam_beta2, adam_eps; /* Alg. 9-11, defaults 0.9, 0.999, 1e-8 */
    int track_gap;   /* maintain m and snapshots in the non-GA modes too */
    int gap_scope;   /* ga_gap_scope, default GA_GAP_PARAMETER */
    uint32_t n_layers;                 /* GA_GAP_LAYER: number of layers */
    const uint64_t* host_layer_sizes;  /* GA_GAP_LAYER: n_layers sizes (each > 0) summing to N; read during
                                          ga_workspace_bytes_ex / ga_create_ex only */
    int nesterov;    /* MOMENTUM family: Nesterov form of the step (Sec. 6 trains with NAG; the paper
                        prints the masters in heavy-ball form only):
                          v = gamma * v + ghat ;  d = ghat + gamma * v ;  theta = theta - lr * d,
                        and Alg. 14 follows d.  Default 0 (heavy ball, as printed). */
} ga_config;

/* ------------------------------------------------------------------ host only
 * These touch no device and need no context. */

/* Defaults listed at ga_config (N and n_workers are set to 0). */
void ga_config_init(ga_config* cfg);


/* Arrival order of n_workers simulated workers (App. C.1: FIFO master).  All
 * workers start at time 0; worker w's n-th iteration takes a time drawn from
 * `dist` by a counter-based generator keyed (seed, w, n), in double; arrivals
 * are served in order of finish time, ties to the lowest id; the update takes
 * no time.  Writes T worker ids to host_schedule.  sigma is used by
 * GA_DIST_LOGNORMAL and GA_DIST_HETERO only. */
int ga_simulate_schedule(uint32_t n_workers, uint64_t T, int dist, double sigma, uint64_t seed,
                         uint32_t* host_schedule);

/* The same for any time model; host_finish_times (optional, T doubles)
 * receives the finish time of every arrival. */
int ga_simulate_schedule_ex(uint32_t n_workers, uint64_t T, const ga_time_model* model, uint64_t seed,
                            uint32_t* host_schedule, double* host_finish_times);

/* App. D: wall-clock time to process n_workers * iters batches with batch
 * times from `model` and no communication cost.  SSGD waits in every iteration
 * for the slowest worker; ASGD ends with arrival number n_workers * iters of
 * the FIFO schedule above. */
int ga_simulate_speedup(uint32_t n_workers, uint64_t iters, const ga_time_model* model, uint64_t seed,
                        double* asgd_wall, double* ssgd_wall);

/* Gradual warm-up of App. C.5: the step size starts at eta / n_workers and
 * rises linearly to eta at master step warmup_steps.  Writes eta_k for the T
 * steps k = k0+1 .. k0+T (evaluated in double, rounded to float). */
int ga_warmup_lr(float eta, uint32_t n_workers, uint64_t warmup_steps, uint64_t k0, uint64_t T, float* host_eta);

/* Delay bookkeeping of Alg. 3 / Alg. 5 for T arrivals starting after master
 * step k0: tau_k = k - iter[i]; iter[i] = k.  host_iter (n_workers entries) is
 * read and updated; host_tau receives T delays. */
int ga_delays_from_schedule(uint32_t n_workers, uint64_t T, const uint32_t* host_schedule, uint64_t k0,
                            uint64_t* host_iter, uint64_t* host_tau);

/* The table rows for the same T arrivals: delays as above plus the step size
 * and the Alg. 14 bias correction of each step.  host_iter is read and
 * updated.  host_rows receives T rows. */
int ga_plan_arrivals(uint32_t n_workers, uint64_t T, const uint32_t* host_schedule, uint64_t k0,
                     uint64_t* host_iter, int mode, float eta_k, float beta, ga_arrival* host_rows);

/* ------------------------------------------------------------------ context */

/* Bytes of device workspace a context needs (state, W snapshots, arrival
 * table, reduction partials).  0 if N or n_workers is 0. */
size_t ga_workspace_bytes(uint64_t N, uint32_t n_workers);

/* Create a master (Alg. 2-5 initial state): theta = v = m = 0, every snapshot
 * = theta, iter = [0]*W, k = 0, eta_k = eta_max = eta, beta = 0.999,
 * eps = 1e-8 (App. C.6), gap tracking off.  dev_workspace: 256-byte aligned,
 * at least ga_workspace_bytes(N, n_workers).  hip_stream: a hipStream_t (may
 * be null for the default stream).  Enqueues the fills of the state.
 * Errors: GA_ERR_ARG for N = 0, n_workers = 0, eta <= 0 or non-finite,
 * |gamma| >= 1 (negative gamma is legal, App. C.9), unknown mode, null out;
 * GA_ERR_ALIGN for a misaligned or short workspace. */
int ga_create(ga_ctx** out, uint64_t N, uint32_t n_workers, float eta, float gamma, int mode,
              void* dev_workspace, size_t workspace_bytes, void* hip_stream);

/* The same for any family.  ga_create(N, W, eta, gamma, mode, ...) is
 * ga_create_ex with the other fields at their defaults.  Extra errors:
 * GA_ERR_ARG for an unknown family, GA_MODE_SA_STEP outside MOMENTUM, Adam
 * betas outside [0,1) or adam_eps <= 0. */
size_t ga_workspace_bytes_ex(const ga_config* cfg);
int ga_create_ex(ga_ctx** out, const ga_config* cfg, void* dev_workspace, size_t workspace_bytes, void* hip_stream);

void ga_destroy(ga_ctx* ctx);

/* Alg. 14 constants.  beta in [0,1), eps > 0 (eps = 0 would make C = 0 at the
 * first arrival).  Only before the first arrival (GA_ERR_STATE afterwards). */
int ga_set_beta_eps(ga_ctx* ctx, float beta, float eps);
/* eta_max of Alg. 14 (> 0).  Only before the first arrival. */
int ga_set_eta_max(ga_ctx* ctx, float eta_max);
/* eta_k for the following arrivals (> 0); eta_max is unchanged. */
int ga_set_lr(ga_ctx* ctx, float eta_k);
/* Maintain m in the non-GA modes too, so that ga_diagnostics can report the
 * Gap under SA / ASGD (costs 8 bytes per parameter per arrival).  Only before
 * the first arrival. */
int ga_set_track_gap(ga_ctx* ctx, int on);
/* How many bytes of theta, v, m (theta first) the update kernels of this
 * master keep in the memory-side cache between arrivals: the leading part of
 * the arrays is accessed without the non-temporal hint, everything else is
 * streamed around the cache.  Default 240 MiB of the MI355X's 256 MiB, right
 * for one master per GPU; masters that share a GPU (or share it with other
 * users of that cache) should split it, and 0 streams everything.  A budget
 * above what the cache holds makes the kept lines evict each other and is
 * slower than 0.  Changes no result, only speed; legal at any step. */
int ga_set_resident_bytes(ga_ctx* ctx, uint64_t bytes);
uint64_t ga_get_resident_bytes(const ga_ctx* ctx);
/* theta_0: copy N floats from dev_theta0 into theta and into every snapshot
 * (App. C.1: theta^i = theta_0).  Only before the first arrival. */
int ga_set_theta(ga_ctx* ctx, const float* dev_theta0);

/* One arrival: worker_id delivers dev_grad (N values of grad_dtype).  Host:
 * k += 1, tau = k - iter[i]; device: one fused launch doing the arithmetic in
 * the header comment for all N parameters; host: iter[i] = k, tau recorded.
 * dev_grad needs only the alignment of its element type (a pointer that is
 * not 16-byte aligned takes a slower path).  In the non-GA modes the snapshot
 * is written (and m maintained) only when gap tracking is on: nothing reads
 * them otherwise, and the arrival then moves 20 instead of 36 bytes per
 * parameter. */
int ga_apply(ga_ctx* ctx, uint32_t worker_id, const void* dev_grad, int grad_dtype);

/* A queue of n arrivals whose gradients are all in device memory, applied in
 * order (Alg. 4 / 5 / 3 per arrival, as ga_apply would) by one launch per
 * chunk of up to 8192 arrivals: theta, v and m stay in registers over the
 * chunk and only the gradient and the arriving worker's snapshot move per
 * arrival.  Same results, bit for bit, as n calls of ga_apply.
 *   host_workers   HOST array of n worker ids (a worker may appear more than once)
 *   host_dev_grads HOST array of n DEVICE pointers, each to N values of
 *                  grad_dtype, aligned to four values (16 bytes for GA_F32,
 *                  8 for GA_BF16); read, never written, not owned; they must
 *                  stay unchanged until the stream has finished
 * Parameter-wise Gap only.  Any family and penalty; the context's step size
 * is used for every arrival.  Asynchronous on the context's stream.
 * Errors (nothing is launched and no bookkeeping changes): GA_ERR_ARG (null
 * pointer, unknown dtype, layer-wise or global Gap), GA_ERR_WORKER,
 * GA_ERR_ALIGN; GA_ERR_HIP from a failed upload or launch leaves the arrivals
 * of the chunks already launched applied. */
int ga_apply_queue(ga_ctx* ctx, uint64_t n, const uint32_t* host_workers, const void* const* host_dev_grads,
                   int grad_dtype);

/* T arrivals in the order of host_schedule (worker ids), gradients from src.
 * All arguments are checked before the first arrival (then nothing has
 * changed on error); if a HIP call fails later (GA_ERR_HIP), the arrivals
 * enqueued before it stay applied and recorded: ga_step tells how many. */
int ga_run_schedule(ga_ctx* ctx, const uint32_t* host_schedule, uint64_t T, const ga_grad_source* src);

/* The same with a step size per arrival: arrival a of this call uses
 * eta_k = host_eta[a] (T values, each finite and > 0); eta_max and the step
 * size set by ga_set_lr are not changed.  host_eta may be null (then this is
 * ga_run_schedule). */
int ga_run_schedule_lr(ga_ctx* ctx, const uint32_t* host_schedule, uint64_t T, const ga_grad_source* src,
                       const float* host_eta);

/* Write the quadratic-plus-noise gradient that worker_id would deliver at the
 * next arrival (step k+1) to dev_g_out (N floats, 16-byte aligned).  State is
 * not changed.  src->kind must be GA_SRC_QUADRATIC_NOISE. */
int ga_quadratic_gradient(ga_ctx* ctx, uint32_t worker_id, const ga_grad_source* src, float* dev_g_out);

/* Gap statistics of worker_id as if its gradient arrived next (C from the
 * current m and 1 - beta^k).  Needs m: a GA mode or gap tracking on, else
 * GA_ERR_STATE.  Waits for the stream; host_out is written on return. */
int ga_diagnostics(ga_ctx* ctx, uint32_t worker_id, ga_diag* host_out);

/* The same statistics without waiting: the kernels are enqueued on the
 * context's stream and the finished report is written to dev_out (DEVICE
 * memory, 8-byte aligned, owned by the caller) when they have run; the
 * arrival stream is not stalled.  Same arguments checks and errors as
 * ga_diagnostics, plus GA_ERR_ALIGN for a misaligned dev_out.  The values
 * are those ga_diagnostics reports (same kernels, same summation order). */
int ga_diagnostics_async(ga_ctx* ctx, uint32_t worker_id, ga_diag* dev_out);

/* For callers that cannot allocate (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the Gap statistics of
 * ga_diagnostics for caller-held arrays, with no context and no workspace.
 * The reduction partials live in a static device array of the library
 * (GA_STATIC_SCRATCH_BYTES per GPU, held until the process ends); this call
 * allocates and frees nothing on host or device.
 *   dev_theta, dev_snapshot, dev_m   DEVICE arrays of N floats, 16-byte
 *                    aligned, read only, owned by the caller
 *   N                1 .. GA_STATIC_MAX_N (GA_ERR_ARG beyond it)
 *   k, beta          C is taken with the bias correction 1 / (1 - beta^k)
 *                    (0 for k = 0), i.e. as the arrival after master step k
 *                    would see it; eta_max, eps as in Alg. 14
 *   dev_out          DEVICE ga_diag, 8-byte aligned, written when the two
 *                    kernels have run on hip_stream (hipStream_t, may be null)
 * Asynchronous.  Every call on one GPU uses that GPU's one array: calls that
 * overlap in time on the same GPU (two streams, two threads) race and give
 * wrong statistics; calls on one stream are ordered and safe.  Nothing in the
 * array has to be cleared between calls (each call writes every partial it
 * reads).  The first call on a GPU looks up the array's address; make that
 * call outside stream capture.  Errors: GA_ERR_ARG, GA_ERR_ALIGN, GA_ERR_HIP;
 * the message is read with ga_last_error(NULL). */
#define GA_STATIC_SCRATCH_BYTES 65536u
#define GA_STATIC_MAX_N (1ull << 40)
int ga_gap_statistics_static(const float* dev_theta, const float* dev_snapshot, const float* dev_m, uint64_t N,
                             uint64_t k, float beta, float eta_max, float eps, ga_diag* dev_out, void* hip_stream);

/* Copies of the state, N floats each, to 4-byte aligned device buffers. */
int ga_get_theta(ga_ctx* ctx, float* dev_dst);
int ga_get_v(ga_ctx* ctx, float* dev_dst);
int ga_get_m(ga_ctx* ctx, float* dev_dst);
int ga_get_snapshot(ga_ctx* ctx, uint32_t worker_id, float* dev_dst);
/* Overwrite v, m or one snapshot from N device floats (tests and checkpoint
 * restore; legal at any step). */
int ga_put_theta(ga_ctx* ctx, const float* dev_src);
int ga_put_v(ga_ctx* ctx, const float* dev_src);
int ga_put_m(ga_ctx* ctx, const float* dev_src);
int ga_put_snapshot(ga_ctx* ctx, uint32_t worker_id, const float* dev_src);

/* Generic access to any state array (N floats; worker_id is used by the
 * per-worker arrays only).  GA_ERR_ARG if the family does not have the array. */
int ga_get_array(ga_ctx* ctx, int which, uint32_t worker_id, float* dev_dst);
int ga_put_array(ga_ctx* ctx, int which, uint32_t worker_id, const float* dev_src);

/* GA_GAP_LAYER / GA_GAP_GLOBAL: the Gaps G_p of the most recent arrival, one
 * float per layer (at most max_n are written).  Waits for the stream.
 * GA_ERR_STATE for a parameter-wise context or before the first arrival. */
int ga_get_layer_gaps(ga_ctx* ctx, float* host_out, uint32_t max_n);

/* Host bookkeeping: current step k; iter[W]; the delays tau_k of the most
 * recent arrivals.  The library keeps the delays of the last 1,048,576
 * arrivals (older ones are dropped, so a long-lived master does not grow):
 * ga_get_delays writes the min(max_n, kept) most recent ones, oldest first,
 * and the number kept to n_out (may be null).  host_out may be null when
 * max_n is 0. */
uint64_t ga_step(const ga_ctx* ctx);
int ga_get_iter(const ga_ctx* ctx, uint64_t* host_iter);
int ga_get_delays(const ga_ctx* ctx, uint64_t* host_out, uint64_t max_n, uint64_t* n_out);
/* The configuration the context runs with (as given to ga_create_ex, with
 * eta = eta_max after ga_set_eta_max and beta, eps after ga_set_beta_eps;
 * host_layer_sizes is returned null) and, if eta_k is not null, the current
 * step size set by ga_set_lr.  A checkpoint holds the state, not these: store
 * them beside it and create the resuming context from them, since Alg. 14
 * continues with another C under another eta_max, beta or eps. */
int ga_get_config(const ga_ctx* ctx, ga_config* out, float* eta_k);
/* Restore k and iter[W] (checkpoint resume; the device arrays are restored
 * with the ga_put_* calls).  Every iter[i] must be <= k. */
int ga_set_bookkeeping(ga_ctx* ctx, uint64_t k, const uint64_t* host_iter);

/* Checkpoint.  The device state of a context (theta, v, m, the W snapshots and
 * the family's extra arrays, in the workspace's own padded layout) is
 * ga_state_bytes(ctx) bytes.  ga_export_state copies it to dev_dst (device
 * buffer of at least that size, 16-byte aligned) and writes the host
 * bookkeeping: *k and host_iter[n_workers].  ga_import_state restores both into
 * a context created with the same N, n_workers, family and gap scope
 * (GA_ERR_ARG if `bytes` differs from ga_state_bytes, or an iter[i] > k; the
 * arrays are padded to whole tiles, so contexts whose N differ by less than a
 * tile can have the same size: the caller keeps N with the checkpoint).
 * Hyper-parameters are not part of the checkpoint.  Running on after an
 * import gives bit for bit the trajectory of the uninterrupted run. */
size_t ga_state_bytes(const ga_ctx* ctx);
int ga_export_state(ga_ctx* ctx, void* dev_dst, size_t bytes, uint64_t* k, uint64_t* host_iter);
int ga_import_state(ga_ctx* ctx, const void* dev_src, size_t bytes, uint64_t k, const uint64_t* host_iter);

/* Fill dev_out[0..n) with z(seed, k, j0 + j), the standard-normal noise of the
 * quadratic source.  One Philox4x32-10 block (Salmon et al., SC'11) with
 * counter (floor(j/4), k) and key seed serves parameters 4q..4q+3: words
 * (x0, x1) feed the Box-Muller pair of lanes 0,1 and (x2, x3) that of lanes
 * 2,3; the even lane takes the cosine.  The transform uses float operations
 * only (atanh series for the logarithm, Taylor series for sine and cosine), so
 * it is reproducible bit for bit.  hip_stream as in ga_create. */
int ga_noise_fill(uint64_t seed, uint64_t k, uint64_t j0, uint64_t n, float* dev_out, void* hip_stream);

/* The Box-Muller transform of ga_noise_fill applied to caller-supplied random
 * words: for i < n, (dev_zc[i], dev_zs[i]) = (r cos, r sin) from the word pair
 * (dev_xa[i], dev_xb[i]).  Lets a test sweep every radius input (2^23 values of
 * xa >> 9) and every angle input (2^25 values of xb >> 7) of the generator. */
int ga_box_muller_raw(const uint32_t* dev_xa, const uint32_t* dev_xb, uint64_t n, float* dev_zc, float* dev_zs,
                      void* hip_stream);

/* ------------------------------------------------------------ measurement aids
 * Behind `bench.py --ceiling`.  They run none of the arithmetic above: they
 * measure what the part delivers for the access pattern and the instruction
 * mix of the kernels, so that the roofline fractions quoted for the kernels
 * can be re-derived on any machine.  The caller times them with events on
 * hip_stream.
 *
 * ga_probe_streams: one launch that reads n_read arrays and writes n_write
 *   arrays of n floats at once (element-wise sum of the inputs to every
 *   output), with the 128-bit non-temporal accesses and the launch shape of
 *   the fused update.  host_dev_read / host_dev_write are HOST arrays of
 *   DEVICE pointers (16-byte aligned, at least n floats each; n a multiple of
 *   4).  n_read in {0, 1, 2, 4, 5}, n_write in {0, 1, 2, 4}, not both 0.
 *   Sec. 4.3 makes the update elementwise, which is why a stream count is all
 *   that characterises its memory side: the GA update is 5 reads + 4 writes.
 * ga_probe_streams_ex: the same with the first n_resident (0, 1 or 2) input
 *   arrays and the first n_resident output arrays accessed without the hint,
 *   as the update accesses the part of theta and v that it keeps in the
 *   memory-side cache.  An output may be the input of the same index (an
 *   update in place); other overlaps between arrays give undefined values.
 *   tiled = 1: the first three input and the first three output arrays are
 *   laid out as a master lays out theta, v, m -- interleaved by tiles of 8192
 *   floats, [a0 tile 0 | a1 tile 0 | a2 tile 0 | a0 tile 1 | ...]: pointer i
 *   (i < 3) is the start of array i's tile 0, i.e. base + 8192 i floats of
 *   one buffer of 3 x (n rounded up to 8192) floats.
 * ga_probe_valu: blocks x 256 threads, each issuing iterations x 8 independent
 *   vector instructions of kind `op` (ga_probe_op); dev_out: 4 bytes, written
 *   only formally.  8 x 256 blocks give 8 wavefronts per SIMD on 256 CUs.
 * Errors: GA_ERR_ARG (counts outside the lists, n_resident above 2, null or
 * misaligned pointers, unknown op), GA_ERR_HIP. */
enum ga_probe_op {
    GA_PROBE_FMA = 0,        /* v_fma_f32 */
    GA_PROBE_XOR = 1,        /* v_xor_b32 */
    GA_PROBE_MUL_HI = 2,     /* v_mul_hi_u32 */
    GA_PROBE_MAD_U64 = 3,    /* v_mad_u64_u32 (Philox's 32 x 32 -> 64 products) */
    GA_PROBE_RCP = 4,        /* v_rcp_f32 */
    GA_PROBE_SQRT = 5,       /* v_sqrt_f32 */
    GA_PROBE_DIV_SCALE = 6,  /* v_div_scale_f32 */
    GA_PROBE_DIV_FMAS = 7,   /* v_div_fmas_f32 */
    GA_PROBE_DIV_FIXUP = 8   /* v_div_fixup_f32 (the three helpers of a correctly rounded division) */
};
int ga_probe_streams(uint32_t n_read, uint32_t n_write, uint64_t n, const float* const* host_dev_read,
                     float* const* host_dev_write, void* hip_stream);
int ga_probe_streams_ex(uint32_t n_read, uint32_t n_write, uint32_t n_resident, int tiled, uint64_t n,
                        const float* const* host_dev_read, float* const* host_dev_write, void* hip_stream);
int ga_probe_valu(int op, uint32_t blocks, uint32_t iterations, uint32_t* dev_out, void* hip_stream);

/* Message of the last error on this context ("" if none).  ctx may be null:
 * then the message of the last failed ga_create on this thread. */
const char* ga_last_error(const ga_ctx* ctx);

/* Library version, "major.minor". */
const char* ga_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GA_H */
