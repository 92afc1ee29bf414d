// CPU oracle for the Gap-Aware (GA) parameter-server master update.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
// GPU library is checked against.  It shares no code with the GPU library and
// must never be called from a product path.
//
// What it follows (Barkai, Hakimi, Schuster, "Gap-Aware Mitigation of Gradient
// Staleness", ICLR 2020):
//   * Momentum-ASGD master                         -- Alg. 2 (Sec. 3)
//   * Staleness-Aware master, step-size form       -- Alg. 3 (Sec. 3.1)
//   * Gap-Aware master, parameter-wise Gap         -- Alg. 4, Eq. 5 (Sec. 4.3)
//   * Staleness-Aware-Gradient master              -- Alg. 5 (App. C.1)
//   * C coefficient                                -- Alg. 14 (App. C.6)
//   * DANA / DANA-SA / DANA-GA masters             -- Alg. 6, 7, 8 (App. C.1)
//   * Adam / Adam-SA / Adam-GA masters             -- Alg. 9, 10, 11 (App. C.1)
//   * layer-wise and global Gap                    -- Eq. 4 and Def. 1 (Sec. 4.3)
//   * Nesterov form of the momentum masters        -- Sec. 2 and Sec. 6 name NAG; form: see master_step
//   * task execution times, gamma (CVB) model      -- Alg. 12, 13 (App. C.3)
//   * ASGD-vs-SSGD speed-up simulation             -- App. D
//   * master is a FIFO over worker arrivals        -- App. C.1
// plus two pieces that are not in the paper and are defined by this project's
// synthetic workloads: the counter-based noise generator used by the
// quadratic-plus-noise gradient source, and the arrival-schedule simulator.
//
// Every routine exists for float (the precision the trajectories are compared
// in) and double (used by the tests to pin the float routine to closed forms).
// Floating-point contraction must be off when compiling this file
// (-ffp-contract=off): each line below is one IEEE operation, and fmaf() is
// written out where a fused operation is meant.
//
// Pins (tests/test_oracle_*.py): Philox known-answer vectors; noise transform
// against libm in double; W=1 reduces every mode to heavy-ball momentum with a
// matrix-power closed form; SA harmonic closed form and the two-step identity
// of Sec. 3.1; constant-gradient closed form for C and the Gap (Gap = delay
// when all updates point the same way, remark after Def. 1); scaling
// invariance of the Gap; schedule closed forms (round robin, mean delay = W
// for exponential times); DANA with one worker against a matrix-power closed
// form and with gamma = 0 against the momentum master; Adam with one worker
// against torch.optim.Adam; Adam-SA / Adam-GA steady-state step eta/tau;
// layers of one parameter against the parameter-wise Gap; gamma variates
// against scipy's gamma distribution and the tail probabilities printed in
// App. C.3 (27.9 % / 1 %); speed-up ratios against the values printed in App. D;
// the Nesterov form with one worker against torch.optim.SGD(nesterov=True);
// without momentum every master against delayed gradient descent written on the
// history of iterates (Sec. 2), with sign-preserving monotone descent for every
// penalty; the Gap statistics' counters on hand-set dyadic values that make
// |d|/C exactly 0, 1/2, 1, 2, inf, nan (App. C.8).
// Parity unpinned (the paper fixes nothing to check these against):
//   * the hinge penalty max(1, |d|/C): this project's variant, pinned only by
//     its definition (the paper's form with "+1" replaced);
//   * which vector feeds Alg. 14: Alg. 14 prints v <- gamma v + g with the raw
//     gradient, Alg. 4 keeps g / G in v; here one v, the update vector actually
//     taken, feeds it (for DANA the arriving worker's v_i, for Adam the update
//     m-hat / (sqrt(v-hat) + eps), for the Nesterov form the step direction).
//     A test records how far this is from the printed form;
//   * the Nesterov form beyond one worker.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <queue>
#include <utility>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
// as 1, 2, 3", SC'11).  Ten rounds of two 32x32->64 multiplies, with the key
// bumped by the Weyl constants between rounds.
// ---------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4]) {
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// ---------------------------------------------------------------------------
// Noise z(seed, k, j): standard normal for arrival k (1-based), parameter j.
//
// One Philox block serves parameters 4q..4q+3: counter = (q, k), key = seed.
// Words (x0,x1) make the Box-Muller pair for j%4 in {0,1}, words (x2,x3) the
// pair for j%4 in {2,3}; the even parameter takes the cosine, the odd the sine.
//
// The transform is specified in float operations so that every conforming
// implementation returns the same bits:
//   u1  = (2*(xa>>9)+1) * 2^-24            in (0,1), exact in float
//   ln u1 = (e-24)*ln2 + 2*atanh(s),  s = (t-1)/(t+1),  u1*2^24 = t*2^e,
//           t in [sqrt(1/2), sqrt(2)),  atanh by its Taylor series to s^9
//   r   = sqrt(-2 ln u1)
//   angle = q*pi/2 + phi,  q = xb>>30,  phi = h*pi/2,
//           h = (2*((xb>>7)&0x7FFFFF)+1 - 2^23) * 2^-24   in (-1/2, 1/2)
//   sin(phi), cos(phi) by their Taylor series to phi^9 / phi^10
//   z   = r*cos(angle)  or  r*sin(angle)
// ---------------------------------------------------------------------------
struct NoiseBits {
    uint32_t xa, xb;
    int odd;
};

NoiseBits noise_bits(uint64_t seed, uint64_t k, uint64_t j) {
    const uint64_t q = j >> 2;
    const uint32_t ctr[4] = {(uint32_t)q, (uint32_t)(q >> 32), (uint32_t)k, (uint32_t)(k >> 32)};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t x[4];
    philox4x32_10(ctr, key, x);
    const int pair = (int)((j >> 1) & 1);
    NoiseBits b;
    b.xa = x[2 * pair];
    b.xb = x[2 * pair + 1];
    b.odd = (int)(j & 1);
    return b;
}

float box_muller_f32(const NoiseBits& b);

float noise_z_f32(uint64_t seed, uint64_t k, uint64_t j) {
    return box_muller_f32(noise_bits(seed, k, j));
}

// The transform on one word pair; b.odd selects the sine.
float box_muller_f32(const NoiseBits& b) {
    // radius
    const uint32_t M = 2u * (b.xa >> 9) + 1u;          // odd, below 2^24
    int e;
    float t = std::frexp((float)M, &e);                // M = t * 2^e, t in [1/2, 1)
    if (t < 0.70710678f) {
        t = 2.0f * t;
        e -= 1;
    }
    const float E = (float)(e - 24);
    const float num = t - 1.0f;
    const float den = t + 1.0f;
    const float s = num / den;
    const float s2 = s * s;
    float P = fmaf(s2, 1.0f / 9.0f, 1.0f / 7.0f);
    P = fmaf(s2, P, 1.0f / 5.0f);
    P = fmaf(s2, P, 1.0f / 3.0f);
    const float s3 = s * s2;
    const float L = fmaf(s3, P, s);                    // atanh(s)
    const float twoL = 2.0f * L;
    const float lnu = fmaf(E, 0.693147180559945f, twoL);
    const float r = std::sqrt(-2.0f * lnu);

    // angle
    const uint32_t quad = b.xb >> 30;
    const int32_t hi = (int32_t)(2u * ((b.xb >> 7) & 0x7FFFFFu) + 1u) - (1 << 23);
    const float h = (float)hi * 5.9604644775390625e-8f;   // 2^-24
    const float phi = h * 1.5707963267948966f;
    const float p2 = phi * phi;
    float S = fmaf(p2, 1.0f / 362880.0f, -1.0f / 5040.0f);
    S = fmaf(p2, S, 1.0f / 120.0f);
    S = fmaf(p2, S, -1.0f / 6.0f);
    const float p3 = phi * p2;
    const float sn = fmaf(p3, S, phi);
    float Cc = fmaf(p2, -1.0f / 3628800.0f, 1.0f / 40320.0f);
    Cc = fmaf(p2, Cc, -1.0f / 720.0f);
    Cc = fmaf(p2, Cc, 1.0f / 24.0f);
    Cc = fmaf(p2, Cc, -0.5f);
    const float cs = fmaf(p2, Cc, 1.0f);

    float ca, sa;                                      // cos, sin of the full angle
    switch (quad) {
        case 0:  ca = cs;  sa = sn;  break;
        case 1:  ca = -sn; sa = cs;  break;
        case 2:  ca = -cs; sa = -sn; break;
        default: ca = sn;  sa = -cs; break;
    }
    return r * (b.odd ? sa : ca);
}

// The same draw evaluated from the Box-Muller definition in double with libm:
// what noise_z_f32 approximates.  Used only to pin noise_z_f32.
double noise_z_ref(uint64_t seed, uint64_t k, uint64_t j) {
    const NoiseBits b = noise_bits(seed, k, j);
    const double u1 = (double)(2u * (b.xa >> 9) + 1u) / 16777216.0;
    const double r = std::sqrt(-2.0 * std::log(u1));
    const double quad = (double)(b.xb >> 30);
    const double h = ((double)(2u * ((b.xb >> 7) & 0x7FFFFFu) + 1u) - 8388608.0) / 16777216.0;
    const double angle = (quad + h) * 1.5707963267948966192313216916398;
    return r * (b.odd ? std::sin(angle) : std::cos(angle));
}

// ---------------------------------------------------------------------------
// Iteration-time draws for the arrival-schedule simulator.  All in double.
// A draw depends only on (seed, worker, iteration index): counter-based, so
// the order in which draws are requested does not matter.
// ---------------------------------------------------------------------------
enum TimeDist {
    DIST_EXP = 0,         // Exp(mean 1), i.i.d. per iteration
    DIST_LOGNORMAL = 1,   // exp(sigma * z), i.i.d. per iteration
    DIST_HETERO = 2,      // per-worker mean exp(sigma * z_w), times Exp(1) per iteration
    DIST_GAMMA_HOMO = 3,  // Alg. 12: homogeneous machines
    DIST_GAMMA_HETERO = 4 // Alg. 13: heterogeneous machines
};

// Parameters of the time model.  sigma: lognormal / hetero.  mean, v_mach, v_task: gamma model
// (mu_task = mu_mach = mean; alpha_task = 1/v_task^2; alpha_mach = 1/v_mach^2; App. C.3).
struct TimeModel {
    int dist;
    double sigma, mean, v_mach, v_task;
};

const uint32_t TAG_TIME = 0x54494D45u;   // counter word 3 of an iteration draw
const uint32_t TAG_MEAN = 0x4D45414Eu;   // counter word 3 of a per-worker draw
const uint32_t TAG_GAMMA = 0x47000000u;  // counter word 3 of a gamma draw: + 65536 * kind + attempt

double u53(uint32_t lo, uint32_t hi) {
    const uint64_t r = ((uint64_t)hi << 32) | lo;
    return (double)(r >> 11) * (1.0 / 9007199254740992.0);   // [0,1)
}

double std_normal_from(const uint32_t x[4]) {
    const double u = u53(x[0], x[1]);
    const double w = u53(x[2], x[3]);
    return std::sqrt(-2.0 * std::log1p(-u)) * std::cos(6.283185307179586476925286766559 * w);
}

double worker_mean(double sigma, uint64_t seed, uint32_t w) {
    const uint32_t ctr[4] = {w, 0u, 0u, TAG_MEAN};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t x[4];
    philox4x32_10(ctr, key, x);
    return std::exp(sigma * std_normal_from(x));
}

// G(alpha, scale), alpha >= 1: Marsaglia and Tsang, "A simple method for generating gamma
// variables" (ACM TOMS 26, 2000).  Attempt a of draw (c0, c1, c2, kind) uses the Philox block
// with counter word 3 = TAG_GAMMA + 65536*kind + a: (x0,x1) and x2 give the normal
// (Box-Muller radius and angle), x3 the acceptance uniform.
double gamma_draw(double alpha, double scale, uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t kind) {
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    const double d = alpha - 1.0 / 3.0;
    const double c = 1.0 / std::sqrt(9.0 * d);
    for (uint32_t attempt = 0; attempt < 65536; ++attempt) {
        const uint32_t ctr[4] = {c0, c1, c2, TAG_GAMMA + 65536u * kind + attempt};
        uint32_t x[4];
        philox4x32_10(ctr, key, x);
        const double radius = std::sqrt(-2.0 * std::log1p(-u53(x[0], x[1])));
        const double z = radius * std::cos(6.283185307179586476925286766559 * (((double)x[2] + 0.5) / 4294967296.0));
        const double ua = ((double)x[3] + 0.5) / 4294967296.0;
        double v = 1.0 + c * z;
        if (v <= 0.0) continue;
        v = v * v * v;
        if (std::log(ua) < 0.5 * z * z + d - d * v + d * std::log(v)) return d * v * scale;
    }
    return std::numeric_limits<double>::quiet_NaN();
}

// Alg. 12: q = G(alpha_task, mu/alpha_task), one draw for the whole run.
double gamma_homo_q(const TimeModel& tm, uint64_t seed) {
    const double alpha_task = 1.0 / (tm.v_task * tm.v_task);
    return gamma_draw(alpha_task, tm.mean / alpha_task, seed, 0, 0, 0, 1);
}
// Alg. 13: p[j] = G(alpha_mach, mu/alpha_mach), one draw per machine.
double gamma_hetero_p(const TimeModel& tm, uint64_t seed, uint32_t w) {
    const double alpha_mach = 1.0 / (tm.v_mach * tm.v_mach);
    return gamma_draw(alpha_mach, tm.mean / alpha_mach, seed, w, 0, 0, 2);
}

double iteration_time(const TimeModel& tm, uint64_t seed, uint32_t w, uint64_t n) {
    if (tm.dist == DIST_GAMMA_HOMO) {          // time = G(alpha_mach, q/alpha_mach)
        const double alpha_mach = 1.0 / (tm.v_mach * tm.v_mach);
        return gamma_draw(alpha_mach, gamma_homo_q(tm, seed) / alpha_mach, seed, (uint32_t)n, (uint32_t)(n >> 32), w, 0);
    }
    if (tm.dist == DIST_GAMMA_HETERO) {        // time = G(alpha_task, p[w]/alpha_task)
        const double alpha_task = 1.0 / (tm.v_task * tm.v_task);
        return gamma_draw(alpha_task, gamma_hetero_p(tm, seed, w) / alpha_task, seed, (uint32_t)n, (uint32_t)(n >> 32), w, 0);
    }
    const uint32_t ctr[4] = {(uint32_t)n, (uint32_t)(n >> 32), w, TAG_TIME};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t x[4];
    philox4x32_10(ctr, key, x);
    switch (tm.dist) {
        case DIST_EXP:
            return -std::log1p(-u53(x[0], x[1]));
        case DIST_LOGNORMAL:
            return std::exp(tm.sigma * std_normal_from(x));
        case DIST_HETERO:
            return worker_mean(tm.sigma, seed, w) * (-std::log1p(-u53(x[0], x[1])));
        default:
            return std::numeric_limits<double>::quiet_NaN();
    }
}

// ---------------------------------------------------------------------------
// Arrival schedule: all workers start at time 0 holding the initial
// parameters; a worker's n-th iteration takes iteration_time(w, n); the master
// serves arrivals in order of finish time (FIFO, App. C.1), ties to the lowest
// worker id; the update itself takes no time and the worker restarts at once.
// ---------------------------------------------------------------------------
void simulate_schedule(uint32_t W, uint64_t T, const TimeModel& tm, uint64_t seed,
                       uint32_t* schedule, double* finish_times) {
    typedef std::pair<double, uint32_t> Ev;   // (finish time, worker)
    std::priority_queue<Ev, std::vector<Ev>, std::greater<Ev>> pq;
    std::vector<uint64_t> n_done(W, 0);
    for (uint32_t w = 0; w < W; ++w) pq.push(Ev(iteration_time(tm, seed, w, 0), w));
    for (uint64_t k = 0; k < T; ++k) {
        const Ev ev = pq.top();
        pq.pop();
        const uint32_t w = ev.second;
        schedule[k] = w;
        if (finish_times) finish_times[k] = ev.first;
        n_done[w] += 1;
        pq.push(Ev(ev.first + iteration_time(tm, seed, w, n_done[w]), w));
    }
}

// Delay bookkeeping of Alg. 3 / Alg. 5: iter = [0]*W; at arrival k (1-based)
// of worker i: tau_k = k - iter[i]; iter[i] = k.
void delays_from_schedule(uint32_t W, uint64_t T, const uint32_t* schedule, uint64_t k0,
                          uint64_t* iter, uint64_t* tau) {
    (void)W;
    for (uint64_t a = 0; a < T; ++a) {
        const uint64_t k = k0 + a + 1;
        const uint32_t i = schedule[a];
        tau[a] = k - iter[i];
        iter[i] = k;
    }
}

// App. D: wall-clock time to process W*iters batches.  SSGD: every iteration waits for the slowest
// of the W workers.  ASGD: the master serves arrivals as they come (the schedule above); the run
// ends with arrival number W*iters.  Batch times only, no communication.
void speedup_times(uint32_t W, uint64_t iters, const TimeModel& tm, uint64_t seed, double* asgd_wall,
                   double* ssgd_wall) {
    double sync = 0.0;
    for (uint64_t i = 0; i < iters; ++i) {
        double slowest = 0.0;
        for (uint32_t w = 0; w < W; ++w) slowest = std::fmax(slowest, iteration_time(tm, seed, w, i));
        sync += slowest;
    }
    typedef std::pair<double, uint32_t> Ev;
    std::priority_queue<Ev, std::vector<Ev>, std::greater<Ev>> pq;
    std::vector<uint64_t> n_done(W, 0);
    for (uint32_t w = 0; w < W; ++w) pq.push(Ev(iteration_time(tm, seed, w, 0), w));
    double last = 0.0;
    for (uint64_t k = 0; k < (uint64_t)W * iters; ++k) {
        const Ev ev = pq.top();
        pq.pop();
        last = ev.first;
        n_done[ev.second] += 1;
        pq.push(Ev(ev.first + iteration_time(tm, seed, ev.second, n_done[ev.second]), ev.second));
    }
    *asgd_wall = last;
    *ssgd_wall = sync;
}

// ---------------------------------------------------------------------------
// The master update.
// ---------------------------------------------------------------------------
enum Mode { MODE_ASGD = 0, MODE_SA = 1, MODE_SA_STEP = 2, MODE_GA = 3, MODE_GA_HINGE = 4 };

template <typename R>
struct Hyper {
    R eta_k;     // step size of this arrival
    R eta_max;   // Alg. 14 "Require"
    R gamma;     // momentum coefficient
    R beta;      // Alg. 14 decay (called beta_1 there)
    R eps;       // Alg. 14 epsilon
};

// 1 / (1 - beta^k), evaluated in double and rounded once to R: Alg. 14's bias
// correction m-hat_k = m_k / (1 - beta^k) is applied as a multiplication by
// this factor (the paper does not fix the rounding).  k = 0 (nothing received
// yet, m_0 = 0, "0/0"): the factor is taken as 0, so that m-hat_0 = 0.
template <typename R>
R inverse_bias_correction(R beta, uint64_t k) {
    if (k == 0) return (R)0;
    return (R)(1.0 / (1.0 - std::pow((double)beta, (double)k)));
}

// C_{k-1}: the coefficient as Alg. 14 leaves it after arrival k-1, from the
// stored biased moment m_{k-1}.
template <typename R>
R coefficient_C(R m, R inv_bc_prev, R eta_max, R eps) {
    const R m_hat = m * inv_bc_prev;
    const R root = std::sqrt(m_hat);
    const R sum = root + eps;
    return eta_max * sum;
}

// One arrival of worker i (gradient g, delay tau, master step k >= 1) applied to
// all n parameters.  snap_i is theta^i: what the master last sent to worker i.
// nesterov: the experiments of Sec. 6 use "a NAG optimizer" but the paper writes
// every master in heavy-ball form; the Nesterov form taken here is the common one,
//   v <- gamma v + g-hat ;  d = g-hat + gamma v ;  theta <- theta - eta d,
// and Alg. 14 then follows d, the step actually taken.
template <typename R>
void master_step(uint64_t n, R* theta, R* v, R* m, R* snap_i, const R* g, int mode, uint64_t k,
                 uint64_t tau, const Hyper<R>& h, int track_gap, int nesterov = 0) {
    const bool gap_mode = (mode == MODE_GA || mode == MODE_GA_HINGE);
    const bool keep_m = gap_mode || track_gap;
    const R inv_bc_prev = inverse_bias_correction<R>(h.beta, k - 1);
    const R one_minus_beta = (R)1 - h.beta;
    const R tau_r = (R)tau;
    const R lr = (mode == MODE_SA_STEP) ? h.eta_k / tau_r : h.eta_k;   // Alg. 3
#pragma omp parallel for schedule(static)
    for (int64_t jj = 0; jj < (int64_t)n; ++jj) {
        const uint64_t j = (uint64_t)jj;
        R g_hat = g[j];
        if (gap_mode) {
            const R diff = theta[j] - snap_i[j];
            const R delta = std::fabs(diff);
            const R C = coefficient_C<R>(m[j], inv_bc_prev, h.eta_max, h.eps);
            const R g_raw = delta / C;
            const R G = (mode == MODE_GA) ? (R)1 + g_raw          // Alg. 4 / Eq. 5
                                          : std::fmax((R)1, g_raw);
            g_hat = g[j] / G;
        } else if (mode == MODE_SA) {
            g_hat = g[j] / tau_r;                                  // Alg. 5
        }
        const R gv = h.gamma * v[j];
        const R v_new = gv + g_hat;                                // v_{k+1}
        R dir = v_new;                                             // update vector
        if (nesterov) {
            const R look = h.gamma * v_new;
            dir = g_hat + look;
        }
        const R step = lr * dir;
        const R theta_new = theta[j] - step;                       // theta_{k+1}
        v[j] = v_new;
        theta[j] = theta_new;
        if (keep_m) {                                              // Alg. 14
            const R bm = h.beta * m[j];
            const R vv = dir * dir;
            const R add = one_minus_beta * vv;
            m[j] = bm + add;
        }
        snap_i[j] = theta_new;                                     // save and send
    }
}

// ---------------------------------------------------------------------------
// Penalty shared by the three families: the factor the gradient is divided by.
//   GA modes: G from the parameter-wise Gap (Eq. 5) with C_{k-1} (Alg. 14)
//   SA:       tau_k                              (Alg. 5 / 7 / 10)
//   else:     1
// ---------------------------------------------------------------------------
template <typename R>
R penalty(int mode, R theta, R snap, R c_state, R inv_bc_prev, R tau_r, R eta_max, R eps) {
    if (mode == MODE_GA || mode == MODE_GA_HINGE) {
        const R diff = theta - snap;
        const R delta = std::fabs(diff);
        const R C = coefficient_C<R>(c_state, inv_bc_prev, eta_max, eps);
        const R g_raw = delta / C;
        return (mode == MODE_GA) ? (R)1 + g_raw : std::fmax((R)1, g_raw);
    }
    if (mode == MODE_SA) return tau_r;
    return (R)1;
}

// DANA masters (Alg. 6 / 7 / 8): one momentum vector per worker, v^i; the
// master steps with the arriving worker's momentum and hands the worker a
// look-ahead estimate theta - eta*gamma*sum_j v^j.  vsum = sum_j v^j is kept
// incrementally.  m is the Alg. 14 state, fed with the step actually taken (v^i).
template <typename R>
void dana_step(uint64_t n, R* theta, R* v_i, R* vsum, R* m, R* snap_i, const R* g, int mode, uint64_t k,
               uint64_t tau, const Hyper<R>& h, int track_gap) {
    const bool gap_mode = (mode == MODE_GA || mode == MODE_GA_HINGE);
    const bool keep_m = gap_mode || track_gap;
    const R inv_bc_prev = inverse_bias_correction<R>(h.beta, k - 1);
    const R one_minus_beta = (R)1 - h.beta;
    const R tau_r = (R)tau;
    const R eta_gamma = h.eta_k * h.gamma;
#pragma omp parallel for schedule(static)
    for (int64_t jj = 0; jj < (int64_t)n; ++jj) {
        const uint64_t j = (uint64_t)jj;
        R g_hat = g[j];
        if (gap_mode || mode == MODE_SA) {
            const R G = penalty<R>(mode, theta[j], snap_i[j], m[j], inv_bc_prev, tau_r, h.eta_max, h.eps);
            g_hat = g[j] / G;
        }
        const R v_old = v_i[j];
        const R gv = h.gamma * v_old;
        const R v_new = gv + g_hat;                 // v^i <- gamma v^i + g / G
        const R step = h.eta_k * v_new;
        const R theta_new = theta[j] - step;        // theta_{k+1} <- theta_k - eta v^i
        const R less = vsum[j] - v_old;
        const R sum_new = less + v_new;             // sum_j v^j with the new v^i
        v_i[j] = v_new;
        theta[j] = theta_new;
        vsum[j] = sum_new;
        if (keep_m) {
            const R bm = h.beta * m[j];
            const R vv = v_new * v_new;
            const R add = one_minus_beta * vv;
            m[j] = bm + add;
        }
        const R ahead = eta_gamma * sum_new;
        snap_i[j] = theta_new - ahead;              // theta^i <- theta_{k+1} - eta gamma sum_j v^j
    }
}

template <typename R>
struct AdamHyper {
    R beta1, beta2, eps;
};

// Adam masters (Alg. 9 / 10 / 11).  The penalty goes on the first moment only
// (App. C.1): m1 <- beta1 m1 + ((1-beta1)/G) g ; v2 <- beta2 v2 + (1-beta2) g^2.
// u = m1-hat / (sqrt(v2-hat) + eps) is the update vector; theta <- theta - eta_k u.
// The Alg. 14 state c follows u (the step the parameters actually take).
template <typename R>
void adam_step(uint64_t n, R* theta, R* m1, R* v2, R* c, R* snap_i, const R* g, int mode, uint64_t k,
               uint64_t tau, const Hyper<R>& h, const AdamHyper<R>& ah, int track_gap) {
    const bool gap_mode = (mode == MODE_GA || mode == MODE_GA_HINGE);
    const bool keep_c = gap_mode || track_gap;
    const R inv_bc_prev = inverse_bias_correction<R>(h.beta, k - 1);
    const R one_minus_beta = (R)1 - h.beta;
    const R omb1 = (R)1 - ah.beta1;
    const R omb2 = (R)1 - ah.beta2;
    const R inv_bc1 = inverse_bias_correction<R>(ah.beta1, k);
    const R inv_bc2 = inverse_bias_correction<R>(ah.beta2, k);
    const R tau_r = (R)tau;
#pragma omp parallel for schedule(static)
    for (int64_t jj = 0; jj < (int64_t)n; ++jj) {
        const uint64_t j = (uint64_t)jj;
        R coef = omb1;
        if (gap_mode || mode == MODE_SA) {
            const R G = penalty<R>(mode, theta[j], snap_i[j], c[j], inv_bc_prev, tau_r, h.eta_max, h.eps);
            coef = omb1 / G;                        // (1 - beta1) / G_k
        }
        const R b1m = ah.beta1 * m1[j];
        const R cg = coef * g[j];
        const R m1_new = b1m + cg;
        const R b2v = ah.beta2 * v2[j];
        const R gg = g[j] * g[j];
        const R add2 = omb2 * gg;
        const R v2_new = b2v + add2;
        const R m1_hat = m1_new * inv_bc1;
        const R v2_hat = v2_new * inv_bc2;
        const R root = std::sqrt(v2_hat);
        const R den = root + ah.eps;
        const R u = m1_hat / den;
        const R step = h.eta_k * u;
        const R theta_new = theta[j] - step;
        m1[j] = m1_new;
        v2[j] = v2_new;
        theta[j] = theta_new;
        if (keep_c) {
            const R bc = h.beta * c[j];
            const R uu = u * u;
            const R add = one_minus_beta * uu;
            c[j] = bc + add;
        }
        snap_i[j] = theta_new;
    }
}

// ---------------------------------------------------------------------------
// Layer-wise Gap (Eq. 4) and, with a single layer, the global Gap (Def. 1):
//   G_p = ||theta_p - theta^i_p|| / C_p + 1,   one penalty per layer p,
// applied to every gradient element of that layer (Alg. 4 otherwise).
// C_p = eta_max (sqrt(sum_{j in p} m-hat_j) + eps): the Alg. 14 estimate of
// E[v_j^2] summed over the layer estimates E||v_p||^2.
// Norms are accumulated in double and rounded once to R.
// layer_sizes: P contiguous layers covering the n parameters.  gaps_out (P
// values, optional) receives G_p.
// ---------------------------------------------------------------------------
template <typename R>
void master_step_layerwise(uint64_t n, R* theta, R* v, R* m, R* snap_i, const R* g, const uint64_t* layer_sizes,
                           uint32_t P, int mode, uint64_t k, const Hyper<R>& h, R* gaps_out, int nesterov) {
    const R inv_bc_prev = inverse_bias_correction<R>(h.beta, k - 1);
    const R one_minus_beta = (R)1 - h.beta;
    uint64_t start = 0;
    for (uint32_t p = 0; p < P; ++p) {
        const uint64_t end = start + layer_sizes[p];
        double dist2 = 0.0, msum = 0.0;
        for (uint64_t j = start; j < end; ++j) {
            const R diff = theta[j] - snap_i[j];
            dist2 += (double)diff * (double)diff;
            msum += (double)m[j];
        }
        const R delta = (R)std::sqrt(dist2);                 // ||theta_p - theta^i_p||
        const R m_hat = (R)msum * inv_bc_prev;
        const R root = std::sqrt(m_hat);
        const R sum = root + h.eps;
        const R C = h.eta_max * sum;
        const R g_raw = delta / C;
        const R G = (mode == MODE_GA) ? (R)1 + g_raw : std::fmax((R)1, g_raw);
        if (gaps_out) gaps_out[p] = G;
        for (uint64_t j = start; j < end; ++j) {
            const R g_hat = g[j] / G;
            const R gv = h.gamma * v[j];
            const R v_new = gv + g_hat;
            R dir = v_new;
            if (nesterov) {                                  // see master_step
                const R look = h.gamma * v_new;
                dir = g_hat + look;
            }
            const R step = h.eta_k * dir;
            const R theta_new = theta[j] - step;
            v[j] = v_new;
            theta[j] = theta_new;
            const R bm = h.beta * m[j];
            const R vv = dir * dir;
            const R add = one_minus_beta * vv;
            m[j] = bm + add;
            snap_i[j] = theta_new;
        }
        start = end;
    }
    (void)n;
}

// Quadratic-plus-noise worker gradient (synthetic stand-in for Alg. 1): the
// worker holds theta_w = snap_i and returns
//   g = a * (theta_w - theta_star) + sigma * z(seed, k, j).
// idx (optional) gives the global parameter index of local element j, so that
// a gathered subset of parameters sees the noise of the full-size run.
template <typename R>
void quadratic_gradient(uint64_t n, R* g, const R* snap_i, const R* a, const R* theta_star,
                        const uint64_t* idx, uint64_t seed, uint64_t k, R sigma) {
#pragma omp parallel for schedule(static)
    for (int64_t jj = 0; jj < (int64_t)n; ++jj) {
        const uint64_t j = (uint64_t)jj;
        const uint64_t gj = idx ? idx[j] : j;
        const R z = (R)noise_z_f32(seed, k, gj);
        const R off = snap_i[j] - theta_star[j];
        const R pull = a[j] * off;
        const R noise = sigma * z;
        g[j] = pull + noise;
    }
}

// Gap statistics of worker i against the current master state, as if its
// gradient arrived next (arrival k+1): Graw = |theta - theta^i| / C_k.
// The paper's Gap is Graw + 1.
template <typename R>
void gap_statistics(uint64_t n, const R* theta, const R* m, const R* snap_i, uint64_t k, R beta,
                    R eta_max, R eps, double* sum_graw, uint64_t* n_gt1, uint64_t* n_gt0,
                    uint64_t* n_nonfinite) {
    const R inv_bc = inverse_bias_correction<R>(beta, k);
    double sum = 0.0;
    uint64_t gt1 = 0, gt0 = 0, bad = 0;
    for (uint64_t j = 0; j < n; ++j) {
        const R diff = theta[j] - snap_i[j];
        const R delta = std::fabs(diff);
        const R C = coefficient_C<R>(m[j], inv_bc, eta_max, eps);
        const R g_raw = delta / C;
        if (!std::isfinite(g_raw)) {
            bad += 1;
            continue;
        }
        sum += (double)g_raw;
        if (g_raw > (R)1) gt1 += 1;
        if (g_raw > (R)0) gt0 += 1;
    }
    *sum_graw = sum;
    *n_gt1 = gt1;
    *n_gt0 = gt0;
    *n_nonfinite = bad;
}

// T arrivals with the quadratic-plus-noise source.  snaps is W rows of n.
template <typename R>
void run_quadratic(uint64_t n, uint32_t /*W*/, uint64_t T, const uint32_t* schedule, R* theta, R* v,
                   R* m, R* snaps, const R* a, const R* theta_star, const uint64_t* idx,
                   uint64_t seed, R sigma, int mode, Hyper<R> h, int track_gap, uint64_t* k_io,
                   uint64_t* iter, uint64_t* tau_out) {
    std::vector<R> g(n);
    uint64_t k = *k_io;
    for (uint64_t a_i = 0; a_i < T; ++a_i) {
        const uint32_t i = schedule[a_i];
        k += 1;
        const uint64_t tau = k - iter[i];
        R* snap_i = snaps + (uint64_t)i * n;
        quadratic_gradient<R>(n, g.data(), snap_i, a, theta_star, idx, seed, k, sigma);
        master_step<R>(n, theta, v, m, snap_i, g.data(), mode, k, tau, h, track_gap);
        iter[i] = k;
        if (tau_out) tau_out[a_i] = tau;
    }
    *k_io = k;
}

// T arrivals with precomputed gradient buffers: arrival a uses
// bufs[pick_by_worker ? worker : (k-1) % n_bufs].
template <typename R>
void run_buffers(uint64_t n, uint32_t W, uint64_t T, const uint32_t* schedule, R* theta, R* v,
                 R* m, R* snaps, const R* bufs, uint32_t n_bufs, int pick_by_worker, int mode,
                 Hyper<R> h, int track_gap, uint64_t* k_io, uint64_t* iter, uint64_t* tau_out) {
    (void)W;
    uint64_t k = *k_io;
    for (uint64_t a_i = 0; a_i < T; ++a_i) {
        const uint32_t i = schedule[a_i];
        k += 1;
        const uint64_t tau = k - iter[i];
        const uint64_t b = pick_by_worker ? (uint64_t)i % n_bufs : (k - 1) % n_bufs;
        master_step<R>(n, theta, v, m, snaps + (uint64_t)i * n, bufs + b * n, mode, k, tau, h,
                       track_gap);
        iter[i] = k;
        if (tau_out) tau_out[a_i] = tau;
    }
    *k_io = k;
}

template <typename R>
Hyper<R> make_hyper(double eta_k, double eta_max, double gamma, double beta, double eps) {
    Hyper<R> h;
    h.eta_k = (R)eta_k;
    h.eta_max = (R)eta_max;
    h.gamma = (R)gamma;
    h.beta = (R)beta;
    h.eps = (R)eps;
    return h;
}

}  // namespace

// ---------------------------------------------------------------------------
// C interface (loaded with ctypes by the tests and by the benchmark's CPU leg).
// Hyper-parameters cross as double; the float routines round them to float
// first, which is exact when the caller passes float values.
// ---------------------------------------------------------------------------
extern "C" {

void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    philox4x32_10(ctr, key, out);
}

float orc_noise_z_f32(uint64_t seed, uint64_t k, uint64_t j) { return noise_z_f32(seed, k, j); }
double orc_noise_z_ref(uint64_t seed, uint64_t k, uint64_t j) { return noise_z_ref(seed, k, j); }

void orc_box_muller_raw(const uint32_t* xa, const uint32_t* xb, uint64_t n, float* zc, float* zs) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        NoiseBits b;
        b.xa = xa[i];
        b.xb = xb[i];
        b.odd = 0;
        zc[i] = box_muller_f32(b);
        b.odd = 1;
        zs[i] = box_muller_f32(b);
    }
}

void orc_noise_fill_f32(uint64_t seed, uint64_t k, uint64_t j0, uint64_t n, float* out) {
    for (uint64_t j = 0; j < n; ++j) out[j] = noise_z_f32(seed, k, j0 + j);
}
void orc_noise_fill_ref(uint64_t seed, uint64_t k, uint64_t j0, uint64_t n, double* out) {
    for (uint64_t j = 0; j < n; ++j) out[j] = noise_z_ref(seed, k, j0 + j);
}

double orc_iteration_time(int dist, double sigma, uint64_t seed, uint32_t w, uint64_t n) {
    const TimeModel tm = {dist, sigma, 0.0, 0.0, 0.0};
    return iteration_time(tm, seed, w, n);
}
double orc_iteration_time_gamma(int dist, double mean, double v_mach, double v_task, uint64_t seed, uint32_t w,
                                uint64_t n) {
    const TimeModel tm = {dist, 0.0, mean, v_mach, v_task};
    return iteration_time(tm, seed, w, n);
}
double orc_gamma_draw(double alpha, double scale, uint64_t seed, uint64_t n) {
    return gamma_draw(alpha, scale, seed, (uint32_t)n, (uint32_t)(n >> 32), 0, 3);
}

int orc_simulate_schedule(uint32_t W, uint64_t T, int dist, double sigma, uint64_t seed,
                          uint32_t* schedule, double* finish_times) {
    if (W == 0 || dist < DIST_EXP || dist > DIST_HETERO) return -1;
    const TimeModel tm = {dist, sigma, 0.0, 0.0, 0.0};
    simulate_schedule(W, T, tm, seed, schedule, finish_times);
    return 0;
}
int orc_simulate_schedule_gamma(uint32_t W, uint64_t T, int dist, double mean, double v_mach, double v_task,
                                uint64_t seed, uint32_t* schedule, double* finish_times) {
    if (W == 0 || (dist != DIST_GAMMA_HOMO && dist != DIST_GAMMA_HETERO)) return -1;
    if (!(mean > 0) || !(v_mach > 0 && v_mach <= 1) || !(v_task > 0 && v_task <= 1)) return -1;
    const TimeModel tm = {dist, 0.0, mean, v_mach, v_task};
    simulate_schedule(W, T, tm, seed, schedule, finish_times);
    return 0;
}
int orc_speedup_times(uint32_t W, uint64_t iters, int dist, double mean, double v_mach, double v_task,
                      uint64_t seed, double* asgd_wall, double* ssgd_wall) {
    if (W == 0 || (dist != DIST_GAMMA_HOMO && dist != DIST_GAMMA_HETERO)) return -1;
    const TimeModel tm = {dist, 0.0, mean, v_mach, v_task};
    speedup_times(W, iters, tm, seed, asgd_wall, ssgd_wall);
    return 0;
}

// Schedule from a caller-supplied table of iteration times (row w, column n),
// for hand-made examples.  times has W rows of max_iters entries.
int orc_schedule_from_times(uint32_t W, uint64_t T, const double* times, uint64_t max_iters,
                            uint32_t* schedule) {
    typedef std::pair<double, uint32_t> Ev;
    std::priority_queue<Ev, std::vector<Ev>, std::greater<Ev>> pq;
    std::vector<uint64_t> n_done(W, 0);
    for (uint32_t w = 0; w < W; ++w) pq.push(Ev(times[(uint64_t)w * max_iters], w));
    for (uint64_t k = 0; k < T; ++k) {
        const Ev ev = pq.top();
        pq.pop();
        const uint32_t w = ev.second;
        schedule[k] = w;
        n_done[w] += 1;
        if (n_done[w] >= max_iters) return -1;
        pq.push(Ev(ev.first + times[(uint64_t)w * max_iters + n_done[w]], w));
    }
    return 0;
}

void orc_delays(uint32_t W, uint64_t T, const uint32_t* schedule, uint64_t k0, uint64_t* iter,
                uint64_t* tau) {
    delays_from_schedule(W, T, schedule, k0, iter, tau);
}

void orc_step_f32(uint64_t n, float* theta, float* v, float* m, float* snap_i, const float* g,
                  int mode, uint64_t k, uint64_t tau, double eta_k, double eta_max, double gamma,
                  double beta, double eps, int track_gap) {
    master_step<float>(n, theta, v, m, snap_i, g, mode, k, tau,
                       make_hyper<float>(eta_k, eta_max, gamma, beta, eps), track_gap);
}
void orc_step_f64(uint64_t n, double* theta, double* v, double* m, double* snap_i, const double* g,
                  int mode, uint64_t k, uint64_t tau, double eta_k, double eta_max, double gamma,
                  double beta, double eps, int track_gap) {
    master_step<double>(n, theta, v, m, snap_i, g, mode, k, tau,
                        make_hyper<double>(eta_k, eta_max, gamma, beta, eps), track_gap);
}

void orc_dana_step_f32(uint64_t n, float* theta, float* v_i, float* vsum, float* m, float* snap_i,
                       const float* g, int mode, uint64_t k, uint64_t tau, double eta_k, double eta_max,
                       double gamma, double beta, double eps, int track_gap) {
    dana_step<float>(n, theta, v_i, vsum, m, snap_i, g, mode, k, tau,
                     make_hyper<float>(eta_k, eta_max, gamma, beta, eps), track_gap);
}
void orc_dana_step_f64(uint64_t n, double* theta, double* v_i, double* vsum, double* m, double* snap_i,
                       const double* g, int mode, uint64_t k, uint64_t tau, double eta_k, double eta_max,
                       double gamma, double beta, double eps, int track_gap) {
    dana_step<double>(n, theta, v_i, vsum, m, snap_i, g, mode, k, tau,
                      make_hyper<double>(eta_k, eta_max, gamma, beta, eps), track_gap);
}
void orc_adam_step_f32(uint64_t n, float* theta, float* m1, float* v2, float* c, float* snap_i,
                       const float* g, int mode, uint64_t k, uint64_t tau, double eta_k, double eta_max,
                       double beta, double eps, double beta1, double beta2, double adam_eps, int track_gap) {
    AdamHyper<float> ah = {(float)beta1, (float)beta2, (float)adam_eps};
    adam_step<float>(n, theta, m1, v2, c, snap_i, g, mode, k, tau,
                     make_hyper<float>(eta_k, eta_max, 0.0, beta, eps), ah, track_gap);
}
void orc_adam_step_f64(uint64_t n, double* theta, double* m1, double* v2, double* c, double* snap_i,
                       const double* g, int mode, uint64_t k, uint64_t tau, double eta_k, double eta_max,
                       double beta, double eps, double beta1, double beta2, double adam_eps, int track_gap) {
    AdamHyper<double> ah = {beta1, beta2, adam_eps};
    adam_step<double>(n, theta, m1, v2, c, snap_i, g, mode, k, tau,
                      make_hyper<double>(eta_k, eta_max, 0.0, beta, eps), ah, track_gap);
}

int orc_step_layerwise_f32(uint64_t n, float* theta, float* v, float* m, float* snap_i, const float* g,
                           const uint64_t* layer_sizes, uint32_t P, int mode, uint64_t k, double eta_k,
                           double eta_max, double gamma, double beta, double eps, float* gaps_out, int nesterov) {
    uint64_t total = 0;
    for (uint32_t p = 0; p < P; ++p) total += layer_sizes[p];
    if (total != n || (mode != MODE_GA && mode != MODE_GA_HINGE)) return -1;
    master_step_layerwise<float>(n, theta, v, m, snap_i, g, layer_sizes, P, mode, k,
                                 make_hyper<float>(eta_k, eta_max, gamma, beta, eps), gaps_out, nesterov);
    return 0;
}
int orc_step_layerwise_f64(uint64_t n, double* theta, double* v, double* m, double* snap_i, const double* g,
                           const uint64_t* layer_sizes, uint32_t P, int mode, uint64_t k, double eta_k,
                           double eta_max, double gamma, double beta, double eps, double* gaps_out, int nesterov) {
    uint64_t total = 0;
    for (uint32_t p = 0; p < P; ++p) total += layer_sizes[p];
    if (total != n || (mode != MODE_GA && mode != MODE_GA_HINGE)) return -1;
    master_step_layerwise<double>(n, theta, v, m, snap_i, g, layer_sizes, P, mode, k,
                                  make_hyper<double>(eta_k, eta_max, gamma, beta, eps), gaps_out, nesterov);
    return 0;
}

void orc_step_nag_f32(uint64_t n, float* theta, float* v, float* m, float* snap_i, const float* g,
                      int mode, uint64_t k, uint64_t tau, double eta_k, double eta_max, double gamma,
                      double beta, double eps, int track_gap) {
    master_step<float>(n, theta, v, m, snap_i, g, mode, k, tau,
                       make_hyper<float>(eta_k, eta_max, gamma, beta, eps), track_gap, 1);
}
void orc_step_nag_f64(uint64_t n, double* theta, double* v, double* m, double* snap_i, const double* g,
                      int mode, uint64_t k, uint64_t tau, double eta_k, double eta_max, double gamma,
                      double beta, double eps, int track_gap) {
    master_step<double>(n, theta, v, m, snap_i, g, mode, k, tau,
                        make_hyper<double>(eta_k, eta_max, gamma, beta, eps), track_gap, 1);
}

void orc_quadratic_gradient_f32(uint64_t n, float* g, const float* snap_i, const float* a,
                                const float* theta_star, const uint64_t* idx, uint64_t seed,
                                uint64_t k, double sigma) {
    quadratic_gradient<float>(n, g, snap_i, a, theta_star, idx, seed, k, (float)sigma);
}
void orc_quadratic_gradient_f64(uint64_t n, double* g, const double* snap_i, const double* a,
                                const double* theta_star, const uint64_t* idx, uint64_t seed,
                                uint64_t k, double sigma) {
    quadratic_gradient<double>(n, g, snap_i, a, theta_star, idx, seed, k, sigma);
}

void orc_gap_statistics_f32(uint64_t n, const float* theta, const float* m, const float* snap_i,
                            uint64_t k, double beta, double eta_max, double eps, double* sum_graw,
                            uint64_t* n_gt1, uint64_t* n_gt0, uint64_t* n_nonfinite) {
    gap_statistics<float>(n, theta, m, snap_i, k, (float)beta, (float)eta_max, (float)eps,
                          sum_graw, n_gt1, n_gt0, n_nonfinite);
}
void orc_gap_statistics_f64(uint64_t n, const double* theta, const double* m, const double* snap_i,
                            uint64_t k, double beta, double eta_max, double eps, double* sum_graw,
                            uint64_t* n_gt1, uint64_t* n_gt0, uint64_t* n_nonfinite) {
    gap_statistics<double>(n, theta, m, snap_i, k, beta, eta_max, eps, sum_graw, n_gt1, n_gt0,
                           n_nonfinite);
}

void orc_run_quadratic_f32(uint64_t n, uint32_t W, uint64_t T, const uint32_t* schedule,
                           float* theta, float* v, float* m, float* snaps, const float* a,
                           const float* theta_star, const uint64_t* idx, uint64_t seed,
                           double sigma, int mode, double eta_k, double eta_max, double gamma,
                           double beta, double eps, int track_gap, uint64_t* k_io, uint64_t* iter,
                           uint64_t* tau_out) {
    run_quadratic<float>(n, W, T, schedule, theta, v, m, snaps, a, theta_star, idx, seed,
                         (float)sigma, mode, make_hyper<float>(eta_k, eta_max, gamma, beta, eps),
                         track_gap, k_io, iter, tau_out);
}
void orc_run_quadratic_f64(uint64_t n, uint32_t W, uint64_t T, const uint32_t* schedule,
                           double* theta, double* v, double* m, double* snaps, const double* a,
                           const double* theta_star, const uint64_t* idx, uint64_t seed,
                           double sigma, int mode, double eta_k, double eta_max, double gamma,
                           double beta, double eps, int track_gap, uint64_t* k_io, uint64_t* iter,
                           uint64_t* tau_out) {
    run_quadratic<double>(n, W, T, schedule, theta, v, m, snaps, a, theta_star, idx, seed, sigma,
                          mode, make_hyper<double>(eta_k, eta_max, gamma, beta, eps), track_gap,
                          k_io, iter, tau_out);
}

void orc_run_buffers_f32(uint64_t n, uint32_t W, uint64_t T, const uint32_t* schedule,
                         float* theta, float* v, float* m, float* snaps, const float* bufs,
                         uint32_t n_bufs, int pick_by_worker, int mode, double eta_k,
                         double eta_max, double gamma, double beta, double eps, int track_gap,
                         uint64_t* k_io, uint64_t* iter, uint64_t* tau_out) {
    run_buffers<float>(n, W, T, schedule, theta, v, m, snaps, bufs, n_bufs, pick_by_worker, mode,
                       make_hyper<float>(eta_k, eta_max, gamma, beta, eps), track_gap, k_io, iter,
                       tau_out);
}
void orc_run_buffers_f64(uint64_t n, uint32_t W, uint64_t T, const uint32_t* schedule,
                         double* theta, double* v, double* m, double* snaps, const double* bufs,
                         uint32_t n_bufs, int pick_by_worker, int mode, double eta_k,
                         double eta_max, double gamma, double beta, double eps, int track_gap,
                         uint64_t* k_io, uint64_t* iter, uint64_t* tau_out) {
    run_buffers<double>(n, W, T, schedule, theta, v, m, snaps, bufs, n_bufs, pick_by_worker, mode,
                        make_hyper<double>(eta_k, eta_max, gamma, beta, eps), track_gap, k_io,
                        iter, tau_out);
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
void orc_set_num_threads(int n) {
#ifdef _OPENMP
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}

}  // extern "C"
