/*
 * CPU oracle for DistSim's strategy evaluation.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the yardstick the GPU library is compared with.  It is called by
 * the tests, by the smoke check and by the benchmark's CPU-baseline leg, and by
 * nothing else; the product path never routes through it.  It shares no code,
 * header, table or helper with the HIP sources.
 *
 * What it is: a plain priority-queue discrete-event simulation, one candidate
 * strategy at a time, that follows DistSim's hierarchical modelling (Sec. 4.3)
 * in the paper's order:
 *
 *   1. model-parallel modelling  -- every layer is mapped to its (composed)
 *      event: one computation event when MP = 1, a computation event followed
 *      by an all-reduce event when MP > 1 (Sec. 4.3, "Model Parallelism
 *      Modeling").  A layer with all-to-all bytes gets one more communication
 *      event per pass (workload extension, not in the paper).
 *   2. pipeline modelling (Algorithm 1) -- walk the schedule S: a device takes
 *      the next stage-task of ITS OWN ordered list as soon as it is idle and
 *      the task's input has arrived (Alg. 1's availability test: the data is
 *      there and it is that micro-batch's turn); the task's events run back to back; when it ends, the
 *      point-to-point event towards the neighbouring stage is appended at
 *      t + elapsed.  GPipe and Dapple (early-backward, "1F1B") orders are built
 *      explicitly as per-device lists.
 *   3. data-parallel modelling -- the lists are identical for every DP replica;
 *      an all-reduce event sized by the gradient bytes is appended at the end
 *      of each device's list (Sec. 4.3, "Data Parallelism Modeling").  With a
 *      bucket size the gradient all-reduce is split into buckets that start as
 *      soon as the last micro-batch's backward has produced their bytes
 *      (extension; bucket = 0 gives the paper's single trailing event; the interleaved and
 *      the explicit schedules fill the buckets per device, see there).
 *      Schedule 2 is the asynchronous pipeline of the paper's discussion of new
 *      algorithms (Sec. 7): the Dapple order minus the global synchronisation
 *      event, i.e. no gradient all-reduce event is appended.
 *   4. analysis -- batch (iteration) time = time of the last event; per-stage
 *      computation / communication busy time = sum of the durations of the
 *      events on that device's list; utilisation = busy / batch (Sec. 3.2,
 *      Sec. 5).
 *
 * Only one device per pipeline stage is simulated: Algorithm 1 appends the same
 * entries to all MP devices of a stage, and DP replicas are duplicates.
 *
 * Collective costs (all integer, truncating division, evaluated exactly in this
 * order; link class k = 0 intra-node, 1 inter-node):
 *   p2p(bytes,k)     = alpha_k + bytes / beta_k
 *   allreduce(n,P,k) = alpha_k + (2*(n-1)*P) / (n*beta_k)      ring volume 2(N-1)P/N, Sec. 4.2
 *   alltoall(n,P,k)  = alpha_k + ((n-1)*P) / (n*beta_k)
 * A collective over n = 1 ranks or over 0 bytes is not an event.  Collectives
 * are intra-node iff n <= gpus_per_node (the paper profiles groups of up to 8 devices directly, Sec. 4.2); a
 * stage boundary s|s+1 is intra-node iff floor(s*tp*dp/g) == floor((s+1)*tp*dp/g)
 * (ranks ordered tp fastest, then dp, then pp; Sec. 4.1's intra/inter attribute).
 *
 * Parity pins for every function here live in tests/test_oracle_*.py (closed
 * forms, hand-worked examples in tests/golden, brute-force longest path,
 * invariants, metamorphic relations).  Agreement with the paper's *measured*
 * batch times (Sec. 5) is parity unpinned: it needs the authors' profiled event
 * times and cluster traces.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ST_OK 0
#define ST_INVALID 1
#define ST_RANGE 2
#define MAX_PP 64        /* devices of one pipeline: the interface's bound on pp (a candidate beyond it is
                            invalid).  Nothing else is bounded here: any micro-batch count, any number of
                            virtual stages and any schedule length is simulated.                      */

enum { EV_TASK_DONE = 0, EV_ARRIVE_F = 1, EV_ARRIVE_B = 2, EV_GRAD_READY = 3, EV_AR_DONE = 4 };

typedef struct {
    int64_t t;
    int64_t seq;
    int32_t kind, stage, mb, layer;
} event_t;

typedef struct {
    event_t *a;
    int64_t n, cap, seq;
} heap_t;

static int ev_less(const event_t *x, const event_t *y) {
    if (x->t != y->t) return x->t < y->t;
    return x->seq < y->seq;
}

static void heap_push(heap_t *h, int64_t t, int kind, int stage, int mb, int layer) {
    if (h->n == h->cap) {
        h->cap = h->cap ? 2 * h->cap : 1024;
        h->a = (event_t *)realloc(h->a, (size_t)h->cap * sizeof(event_t));
    }
    event_t e = { t, h->seq++, kind, stage, mb, layer };
    int64_t i = h->n++;
    while (i > 0) {
        int64_t p = (i - 1) / 2;
        if (!ev_less(&e, &h->a[p])) break;
        h->a[i] = h->a[p];
        i = p;
    }
    h->a[i] = e;
}

static event_t heap_pop(heap_t *h) {
    event_t top = h->a[0];
    event_t e = h->a[--h->n];
    int64_t i = 0;
    for (;;) {
        int64_t c = 2 * i + 1;
        if (c >= h->n) break;
        if (c + 1 < h->n && ev_less(&h->a[c + 1], &h->a[c])) c++;
        if (!ev_less(&h->a[c], &e)) break;
        h->a[i] = h->a[c];
        i = c;
    }
    if (h->n > 0) h->a[i] = e;
    return top;
}

/* ---- collective cost events ------------------------------------------------------- */

typedef struct {
    int32_t num_devices, gpus_per_node;
    int64_t alpha[2], beta[2];
    int64_t bucket;
    int32_t p2p_blocking;   /* 1: the p2p event occupies the sender (it is the tail of the stage-task);
                               2: sends queue on their link (one transfer at a time per direction and boundary) */
} cluster_t;

static int64_t p2p_ns(const cluster_t *cl, int64_t bytes, int k) {
    return cl->alpha[k] + (int64_t)((uint64_t)bytes / (uint64_t)cl->beta[k]);
}

static int64_t allreduce_ns(const cluster_t *cl, int64_t n, int64_t bytes) {
    if (n <= 1 || bytes <= 0) return 0;
    int k = n <= cl->gpus_per_node ? 0 : 1;
    return cl->alpha[k] + (int64_t)((2ull * (uint64_t)(n - 1) * (uint64_t)bytes) / ((uint64_t)n * (uint64_t)cl->beta[k]));
}

static int64_t alltoall_ns(const cluster_t *cl, int64_t n, int64_t bytes) {
    if (n <= 1 || bytes <= 0) return 0;
    int k = n <= cl->gpus_per_node ? 0 : 1;
    return cl->alpha[k] + (int64_t)(((uint64_t)(n - 1) * (uint64_t)bytes) / ((uint64_t)n * (uint64_t)cl->beta[k]));
}

/* ---- one candidate ---------------------------------------------------------------- */

typedef struct {
    int32_t L, V;
    const int32_t *variant_tp;
    const int64_t *fc, *bc, *fa, *ba, *act, *grad, *a2a;
} costs_t;

typedef struct {          /* per-thread scratch, grown on demand */
    heap_t heap;
    uint8_t *task_kind;   /* [pp][2m] 0 = forward, 1 = backward */
    int32_t *task_mb;     /* [pp][2m] */
    uint8_t *arrF, *arrB; /* [pp][m] input of F(s,j) / B(s,j) has arrived */
    int64_t cap_tasks, cap_arr;
} scratch_t;

typedef struct {
    int32_t status;
    int64_t batch_ns, num_events;
} result_t;

static void build_schedule(int pp, int m, int sched, uint8_t *kind, int32_t *mb) {
    for (int s = 0; s < pp; s++) {
        uint8_t *k = kind + (int64_t)s * 2 * m;
        int32_t *j = mb + (int64_t)s * 2 * m;
        int n = 0;
        if (sched == 0) {                 /* GPipe: all forwards, then all backwards, FIFO */
            for (int i = 0; i < m; i++) { k[n] = 0; j[n++] = i; }
            for (int i = 0; i < m; i++) { k[n] = 1; j[n++] = i; }
        } else {                          /* Dapple / 1F1B: warm-up, one-forward-one-backward, cool-down */
            int w = pp - 1 - s;
            if (w > m) w = m;
            int f = 0, b = 0;
            for (int i = 0; i < w; i++) { k[n] = 0; j[n++] = f++; }
            while (f < m) {
                k[n] = 0; j[n++] = f++;
                k[n] = 1; j[n++] = b++;
            }
            while (b < m) { k[n] = 1; j[n++] = b++; }
        }
    }
}

static void simulate_one(const costs_t *co, const cluster_t *cl,
                         int32_t dp, int32_t tp, int32_t pp, int32_t m, int sched,
                         const uint8_t *bnd_in /* NULL = uniform */, int64_t bnd_avail /* entries readable at bnd_in */,
                         scratch_t *sc, result_t *res,
                         int64_t *comp_busy, int64_t *comm_busy, double *util, /* [pp] or NULL */
                         int64_t *tl_start, int64_t *tl_end /* [2][pp][m] or NULL */,
                         int64_t *tl_ar /* [2][pp]: start of the first, end of the last all-reduce; or NULL */) {
    const int L = co->L;
    res->status = ST_INVALID;
    res->batch_ns = INT64_MAX;
    res->num_events = 0;

    /* --- validation ("unreachable" configurations, Sec. 6) --- */
    if (dp < 1 || tp < 1 || pp < 1 || m < 1 || (sched != 0 && sched != 1 && sched != 2)) return;
    if ((int64_t)dp * tp * pp != cl->num_devices) return;
    if (pp > L || pp > MAX_PP) return;
    int v = -1;
    for (int i = 0; i < co->V; i++) if (co->variant_tp[i] == tp) { v = i; break; }
    if (v < 0) return;
    int bnd[MAX_PP + 1];
    if (bnd_in) {
        if (bnd_avail < pp + 1) return;               /* the partition would run off the pool */
        for (int s = 0; s <= pp; s++) bnd[s] = bnd_in[s];
        if (bnd[0] != 0 || bnd[pp] != L) return;
        for (int s = 0; s < pp; s++) if (bnd[s + 1] <= bnd[s]) return;
    } else {
        for (int s = 0; s <= pp; s++) bnd[s] = (int)(((int64_t)s * L) / pp);
    }
    const int64_t *fc = co->fc + (int64_t)v * L, *bc = co->bc + (int64_t)v * L;
    const int64_t *fa = co->fa + (int64_t)v * L, *ba = co->ba + (int64_t)v * L;
    const int64_t *act = co->act + (int64_t)v * L, *grad = co->grad + (int64_t)v * L;
    const int64_t *a2a = co->a2a + (int64_t)v * L;

    /* --- point-to-point events of every stage boundary --- */
    int64_t pf[256], pb[256];      /* pf[s]: s -> s+1 activation; pb[s]: s -> s-1 gradient */
    const int64_t g = cl->gpus_per_node;
    for (int s = 0; s < pp; s++) { pf[s] = 0; pb[s] = 0; }
    for (int s = 0; s + 1 < pp; s++) {
        int64_t na = ((int64_t)s * tp * dp) / g, nb = ((int64_t)(s + 1) * tp * dp) / g;
        int k = na == nb ? 0 : 1;
        int64_t bytes = act[bnd[s + 1] - 1];
        pf[s] = p2p_ns(cl, bytes, k);
        pb[s + 1] = p2p_ns(cl, bytes, k);
    }

    /* --- range guard: every timestamp of the pipeline phase is below 2^53 --- */
    {
        unsigned __int128 t1 = 0;
        for (int s = 0; s < pp; s++) {
            for (int l = bnd[s]; l < bnd[s + 1]; l++) {
                t1 += (unsigned __int128)(fc[l] + bc[l]);
                if (tp > 1) t1 += (unsigned __int128)(fa[l] + ba[l]);
                t1 += 2 * (unsigned __int128)alltoall_ns(cl, dp, a2a[l]);
            }
            t1 += (unsigned __int128)(pf[s] + pb[s]);
        }
        if (t1 * (unsigned __int128)m >= ((unsigned __int128)1 << 53)) { res->status = ST_RANGE; return; }
    }
    res->status = ST_OK;

    /* --- scratch --- */
    int64_t ntask = (int64_t)pp * 2 * m, narr = (int64_t)pp * m;
    if (ntask > sc->cap_tasks) {
        sc->cap_tasks = ntask;
        sc->task_kind = (uint8_t *)realloc(sc->task_kind, (size_t)ntask);
        sc->task_mb = (int32_t *)realloc(sc->task_mb, (size_t)ntask * sizeof(int32_t));
    }
    if (narr > sc->cap_arr) {
        sc->cap_arr = narr;
        sc->arrF = (uint8_t *)realloc(sc->arrF, (size_t)narr);
        sc->arrB = (uint8_t *)realloc(sc->arrB, (size_t)narr);
    }
    memset(sc->arrF, 0, (size_t)narr);
    memset(sc->arrB, 0, (size_t)narr);
    build_schedule(pp, m, sched, sc->task_kind, sc->task_mb);
    const int sync = sched != 2;        /* schedule 2: no global synchronisation (gradient all-reduce) event */

    heap_t *h = &sc->heap;
    h->n = 0; h->seq = 0;

    int32_t next[256];
    uint8_t busy[256];
    int64_t cb[256], mb_[256];          /* computation / communication busy */
    int64_t comm_free[256], acc[256];   /* DP communication stream, open bucket bytes */
    int64_t link_f[256], link_b[256];   /* time at which the outgoing forward / backward link is free again */
    for (int s = 0; s < pp; s++) { next[s] = 0; busy[s] = 0; cb[s] = 0; mb_[s] = 0; comm_free[s] = 0; acc[s] = 0; link_f[s] = 0; link_b[s] = 0; }
    int64_t nev = 0, now = 0;
    if (tl_ar) for (int s = 0; s < 2 * pp; s++) tl_ar[s] = -1;
    const int64_t cap = cl->bucket;

/* start the next task of stage s if the device is idle and the input is there */
#define TRY_START(s_) do {                                                              \
        int s__ = (s_);                                                                 \
        if (!busy[s__] && next[s__] < 2 * m) {                                          \
            int64_t ti = (int64_t)s__ * 2 * m + next[s__];                              \
            int kd = sc->task_kind[ti], j = sc->task_mb[ti];                            \
            int ready = kd == 0 ? (s__ == 0 || sc->arrF[(int64_t)s__ * m + j])          \
                                : (s__ == pp - 1 || sc->arrB[(int64_t)s__ * m + j]);    \
            if (ready) {                                                                \
                busy[s__] = 1;                                                          \
                int64_t t = now;                                                        \
                if (tl_start) tl_start[((int64_t)kd * pp + s__) * m + j] = t;           \
                int last_bwd = (kd == 1 && next[s__] == 2 * m - 1);                     \
                if (kd == 0) {                                                          \
                    for (int l = bnd[s__]; l < bnd[s__ + 1]; l++) {                     \
                        t += fc[l]; cb[s__] += fc[l];                                   \
                        if (tp > 1) { t += fa[l]; mb_[s__] += fa[l]; }                  \
                        int64_t x = alltoall_ns(cl, dp, a2a[l]);                        \
                        t += x; mb_[s__] += x;                                          \
                    }                                                                   \
                } else {                                                                \
                    for (int l = bnd[s__ + 1] - 1; l >= bnd[s__]; l--) {                \
                        t += bc[l]; cb[s__] += bc[l];                                   \
                        if (tp > 1) { t += ba[l]; mb_[s__] += ba[l]; }                  \
                        int64_t x = alltoall_ns(cl, dp, a2a[l]);                        \
                        t += x; mb_[s__] += x;                                          \
                        if (last_bwd && cap > 0 && dp > 1 && sync)                      \
                            heap_push(h, t, EV_GRAD_READY, s__, j, l);                  \
                    }                                                                   \
                }                                                                       \
                if (cl->p2p_blocking == 1) {      /* the send runs on the device */     \
                    if (kd == 0 && s__ + 1 < pp) t += pf[s__];                          \
                    if (kd == 1 && s__ > 0) t += pb[s__];                               \
                }                                                                       \
                heap_push(h, t, EV_TASK_DONE, s__, j, kd);                              \
            }                                                                           \
        }                                                                               \
    } while (0)

    for (int s = 0; s < pp; s++) TRY_START(s);       /* t = 0: start of the first stage's first event */

    while (h->n > 0) {
        event_t e = heap_pop(h);
        now = e.t;
        int s = e.stage;
        switch (e.kind) {
        case EV_TASK_DONE: {
            int kd = e.layer, j = e.mb;
            nev++;
            if (tl_end) tl_end[((int64_t)kd * pp + s) * m + j] = now;
            busy[s] = 0;
            next[s]++;
            if (kd == 0 && s + 1 < pp) {            /* (e_comm, t + e.elapsed, m) of Algorithm 1 */
                int64_t arrive = now + pf[s];
                if (cl->p2p_blocking == 1) arrive = now;
                if (cl->p2p_blocking == 2) {         /* the link carries one activation at a time */
                    int64_t depart = now > link_f[s] ? now : link_f[s];
                    arrive = depart + pf[s];
                    link_f[s] = arrive;
                }
                heap_push(h, arrive, EV_ARRIVE_F, s + 1, j, 0);
                mb_[s] += pf[s]; nev++;
            }
            if (kd == 1 && s > 0) {
                int64_t arrive = now + pb[s];
                if (cl->p2p_blocking == 1) arrive = now;
                if (cl->p2p_blocking == 2) {
                    int64_t depart = now > link_b[s] ? now : link_b[s];
                    arrive = depart + pb[s];
                    link_b[s] = arrive;
                }
                heap_push(h, arrive, EV_ARRIVE_B, s - 1, j, 0);
                mb_[s] += pb[s]; nev++;
            }
            if (next[s] == 2 * m && dp > 1 && cap == 0 && sync) {   /* trailing gradient all-reduce */
                int64_t G = 0;
                for (int l = bnd[s]; l < bnd[s + 1]; l++) G += grad[l];
                if (G > 0) {
                    int64_t d = allreduce_ns(cl, dp, G);
                    heap_push(h, now + d, EV_AR_DONE, s, 0, 0);
                    mb_[s] += d;
                    if (tl_ar) { tl_ar[s] = now; tl_ar[pp + s] = now + d; }
                }
            }
            TRY_START(s);
            break;
        }
        case EV_ARRIVE_F:
            sc->arrF[(int64_t)s * m + e.mb] = 1;
            TRY_START(s);
            break;
        case EV_ARRIVE_B:
            sc->arrB[(int64_t)s * m + e.mb] = 1;
            TRY_START(s);
            break;
        case EV_GRAD_READY: {                        /* bucketed, overlapped gradient all-reduce */
            acc[s] += grad[e.layer];
            while (acc[s] >= cap) {
                int64_t d = allreduce_ns(cl, dp, cap);
                int64_t st = comm_free[s] > now ? comm_free[s] : now;
                comm_free[s] = st + d;
                heap_push(h, comm_free[s], EV_AR_DONE, s, 0, 0);
                mb_[s] += d;
                if (tl_ar) { if (tl_ar[s] < 0) tl_ar[s] = st; tl_ar[pp + s] = comm_free[s]; }
                acc[s] -= cap;
            }
            if (e.layer == bnd[s] && acc[s] > 0) {   /* the stage's first layer finishes last */
                int64_t d = allreduce_ns(cl, dp, acc[s]);
                int64_t st = comm_free[s] > now ? comm_free[s] : now;
                comm_free[s] = st + d;
                heap_push(h, comm_free[s], EV_AR_DONE, s, 0, 0);
                mb_[s] += d;
                if (tl_ar) { if (tl_ar[s] < 0) tl_ar[s] = st; tl_ar[pp + s] = comm_free[s]; }
                acc[s] = 0;
            }
            break;
        }
        case EV_AR_DONE:
            nev++;
            break;
        }
    }
#undef TRY_START

    res->batch_ns = now;
    res->num_events = nev;
    for (int s = 0; s < pp; s++) {
        if (comp_busy) comp_busy[s] = cb[s];
        if (comm_busy) comm_busy[s] = mb_[s];
        if (util) util[s] = now > 0 ? (double)cb[s] / (double)now : 0.0;
    }
}

/* ---- entry points (plain C ABI for ctypes; all pointers are host memory) ---------- */

/* ---- schedule 3: interleaved one-forward-one-backward (extension; the paper's discussion of
 * new algorithms, Sec. 7, says a new pipeline algorithm enters through its schedule) ----------
 *
 * Every device holds `vch` model chunks: virtual stage k = c * pp + d is chunk c of device d and
 * owns the layers [bnd[k], bnd[k+1]) of a partition into S = pp * vch parts.  Micro-batches come
 * in groups of pp (m must be a multiple of pp).  The i-th forward of a device works on chunk
 * (i mod (pp vch)) / pp and micro-batch (i / (pp vch)) pp + i mod pp; the i-th backward on chunk
 * vch - 1 - (i mod (pp vch)) / pp and the same micro-batch.  Device d runs
 * W = min(2 (pp - d - 1) + (vch - 1) pp, m vch) forwards first, then alternates forward and
 * backward, then runs the backwards that are left (Narayanan et al., SC 2021, Sec. 2.2.2).
 * A forward of virtual stage k needs the forward of k - 1 for that micro-batch (the edge from
 * the last device back to the first included), a backward the backward of k + 1; the last
 * virtual stage turns a micro-batch around on its own device.  One gradient all-reduce per device
 * over the bytes of all its chunks follows its last backward.  With a bucket size (extension, as
 * for the built-in schedules): a chunk's gradients are complete in its backward of the last
 * micro-batch, layer by layer from its last layer to its first; the device fills its buckets in
 * that order across its chunks, every full bucket is reduced at once, the events queue on the
 * device's communication stream, and what is left after the device's last gradient goes as one more
 * event.  With p2p_blocking == 2 a link is an ordered pair (sending device, receiving device)
 * and carries one transfer at a time, whatever chunks the transfers belong to.
 * Timeline arrays, if given, are [2][S][m] (virtual stage, not device).
 */
static void simulate_interleaved(const costs_t *co, const cluster_t *cl,
                                 int32_t dp, int32_t tp, int32_t pp, int32_t m, int32_t vch,
                                 const uint8_t *bnd_in, int64_t bnd_avail, scratch_t *sc, result_t *res,
                                 int64_t *comp_busy, int64_t *comm_busy, double *util,
                                 int64_t *tl_start, int64_t *tl_end, int64_t *tl_ar) {
    const int L = co->L;
    res->status = ST_INVALID;
    res->batch_ns = INT64_MAX;
    res->num_events = 0;
    if (dp < 1 || tp < 1 || pp < 1 || pp > MAX_PP || m < 1 || vch < 1) return;
    if ((int64_t)dp * tp * pp != cl->num_devices) return;
    if ((int64_t)pp * vch > L || m % pp != 0) return;
    const int S = pp * vch;
    if (bnd_in && bnd_avail < S + 1) return;
    int v = -1;
    for (int i = 0; i < co->V; i++) if (co->variant_tp[i] == tp) { v = i; break; }
    if (v < 0) return;
    int *bnd = (int *)malloc((size_t)(S + 1) * sizeof(int));
    int64_t *pf = (int64_t *)calloc((size_t)S, sizeof(int64_t)), *pb = (int64_t *)calloc((size_t)S, sizeof(int64_t));
    int64_t *link_free = (int64_t *)calloc((size_t)pp * pp, sizeof(int64_t));   /* [sender][receiver]: free again at */
#define FREE_I() do { free(bnd); free(pf); free(pb); free(link_free); } while (0)
    if (bnd_in) {
        int okp = 1;
        for (int k = 0; k <= S; k++) bnd[k] = bnd_in[k];
        if (bnd[0] != 0 || bnd[S] != L) okp = 0;
        for (int k = 0; k < S && okp; k++) if (bnd[k + 1] <= bnd[k]) okp = 0;
        if (!okp) { FREE_I(); return; }
    } else {
        for (int k = 0; k <= S; k++) bnd[k] = (int)(((int64_t)k * L) / S);
    }
    const int64_t *fc = co->fc + (int64_t)v * L, *bc = co->bc + (int64_t)v * L;
    const int64_t *fa = co->fa + (int64_t)v * L, *ba = co->ba + (int64_t)v * L;
    const int64_t *act = co->act + (int64_t)v * L, *grad = co->grad + (int64_t)v * L;
    const int64_t *a2a = co->a2a + (int64_t)v * L;

    /* p2p events of every boundary between virtual stages, by the nodes of the two devices */
    const int64_t g = cl->gpus_per_node;
    for (int k = 0; k + 1 < S; k++) {
        int64_t na = ((int64_t)(k % pp) * tp * dp) / g, nb = ((int64_t)((k + 1) % pp) * tp * dp) / g;
        int cls = na == nb ? 0 : 1;
        int64_t bytes = act[bnd[k + 1] - 1];
        pf[k] = p2p_ns(cl, bytes, cls);
        pb[k + 1] = p2p_ns(cl, bytes, cls);
    }
    {
        unsigned __int128 t1 = 0;
        for (int k = 0; k < S; k++) {
            for (int l = bnd[k]; l < bnd[k + 1]; l++) {
                t1 += (unsigned __int128)(fc[l] + bc[l]);
                if (tp > 1) t1 += (unsigned __int128)(fa[l] + ba[l]);
                t1 += 2 * (unsigned __int128)alltoall_ns(cl, dp, a2a[l]);
            }
            t1 += (unsigned __int128)(pf[k] + pb[k]);
        }
        if (t1 * (unsigned __int128)m >= ((unsigned __int128)1 << 53)) { res->status = ST_RANGE; FREE_I(); return; }
    }
    res->status = ST_OK;

    /* per-device ordered task lists: kind, micro-batch; the virtual stage goes to a third array */
    const int64_t per_dev = 2ll * m * vch;
    int64_t ntask = (int64_t)pp * per_dev, narr = (int64_t)S * m;
    if (ntask > sc->cap_tasks) {
        sc->cap_tasks = ntask;
        sc->task_kind = (uint8_t *)realloc(sc->task_kind, (size_t)ntask);
        sc->task_mb = (int32_t *)realloc(sc->task_mb, (size_t)ntask * sizeof(int32_t));
    }
    if (narr > sc->cap_arr) {
        sc->cap_arr = narr;
        sc->arrF = (uint8_t *)realloc(sc->arrF, (size_t)narr);
        sc->arrB = (uint8_t *)realloc(sc->arrB, (size_t)narr);
    }
    memset(sc->arrF, 0, (size_t)narr);
    memset(sc->arrB, 0, (size_t)narr);
    int32_t *task_vs = (int32_t *)malloc((size_t)ntask * sizeof(int32_t));
    const int64_t nslot = (int64_t)m * vch;
    for (int d = 0; d < pp; d++) {
        uint8_t *kk = sc->task_kind + d * per_dev;
        int32_t *vs = task_vs + d * per_dev;
        int32_t *jj = sc->task_mb + d * per_dev;
        int64_t W = 2ll * (pp - d - 1) + (int64_t)(vch - 1) * pp;
        if (W > nslot) W = nslot;
        int64_t n = 0, f = 0, b = 0;
#define PUT_F(i_) do { int64_t i__ = (i_), w__ = i__ % ((int64_t)pp * vch);                              \
            kk[n] = 0; vs[n] = (int32_t)((w__ / pp) * pp + d);                                            \
            jj[n] = (int32_t)((i__ / ((int64_t)pp * vch)) * pp + w__ % pp); n++; } while (0)
#define PUT_B(i_) do { int64_t i__ = (i_), w__ = i__ % ((int64_t)pp * vch);                              \
            kk[n] = 1; vs[n] = (int32_t)((vch - 1 - w__ / pp) * pp + d);                                  \
            jj[n] = (int32_t)((i__ / ((int64_t)pp * vch)) * pp + w__ % pp); n++; } while (0)
        for (; f < W; f++) PUT_F(f);
        while (f < nslot) { PUT_F(f); f++; PUT_B(b); b++; }
        while (b < nslot) { PUT_B(b); b++; }
#undef PUT_F
#undef PUT_B
    }

    heap_t *h = &sc->heap;
    h->n = 0; h->seq = 0;
    int64_t next[64];
    uint8_t busy[64];
    int64_t cb[64], mb_[64];
    int64_t comm_free[64], acc[64], pend[64];     /* DP communication stream, open bucket bytes, gradients still to come */
    for (int d = 0; d < pp; d++) {
        next[d] = 0; busy[d] = 0; cb[d] = 0; mb_[d] = 0; comm_free[d] = 0; acc[d] = 0; pend[d] = 0;
        for (int c = 0; c < vch; c++) pend[d] += bnd[c * pp + d + 1] - bnd[c * pp + d];
    }
    int64_t nev = 0, now = 0;
    if (tl_ar) for (int d = 0; d < 2 * pp; d++) tl_ar[d] = -1;
    const int64_t cap = cl->bucket;

#define TRY_START_I(d_) do {                                                            \
        int d__ = (d_);                                                                 \
        if (!busy[d__] && next[d__] < per_dev) {                                        \
            int64_t ti = d__ * per_dev + next[d__];                                     \
            int kd = sc->task_kind[ti], j = sc->task_mb[ti], k = task_vs[ti];           \
            int ready = kd == 0 ? (k == 0 || sc->arrF[(int64_t)k * m + j])              \
                                : sc->arrB[(int64_t)k * m + j];                         \
            if (ready) {                                                                \
                busy[d__] = 1;                                                          \
                int64_t t = now;                                                        \
                if (tl_start) tl_start[((int64_t)kd * S + k) * m + j] = t;              \
                if (kd == 0) {                                                          \
                    for (int l = bnd[k]; l < bnd[k + 1]; l++) {                         \
                        t += fc[l]; cb[d__] += fc[l];                                   \
                        if (tp > 1) { t += fa[l]; mb_[d__] += fa[l]; }                  \
                        int64_t x = alltoall_ns(cl, dp, a2a[l]);                        \
                        t += x; mb_[d__] += x;                                          \
                    }                                                                   \
                } else {                                                                \
                    for (int l = bnd[k + 1] - 1; l >= bnd[k]; l--) {                    \
                        t += bc[l]; cb[d__] += bc[l];                                   \
                        if (tp > 1) { t += ba[l]; mb_[d__] += ba[l]; }                  \
                        int64_t x = alltoall_ns(cl, dp, a2a[l]);                        \
                        t += x; mb_[d__] += x;                                          \
                        if (j == m - 1 && cap > 0 && dp > 1)                            \
                            heap_push(h, t, EV_GRAD_READY, k, j, l);                    \
                    }                                                                   \
                }                                                                       \
                if (cl->p2p_blocking == 1) {                                            \
                    if (kd == 0 && k + 1 < S) t += pf[k];                               \
                    if (kd == 1 && k > 0) t += pb[k];                                   \
                }                                                                       \
                heap_push(h, t, EV_TASK_DONE, k, j, kd);                                \
            }                                                                           \
        }                                                                               \
    } while (0)

    for (int d = 0; d < pp; d++) TRY_START_I(d);
    while (h->n > 0) {
        event_t e = heap_pop(h);
        now = e.t;
        int k = e.stage, d = k % pp;
        switch (e.kind) {
        case EV_TASK_DONE: {
            int kd = e.layer, j = e.mb;
            nev++;
            if (tl_end) tl_end[((int64_t)kd * S + k) * m + j] = now;
            busy[d] = 0;
            next[d]++;
            if (kd == 0 && k + 1 < S) {
                int64_t arrive = now + pf[k];
                if (cl->p2p_blocking == 1) arrive = now;
                if (cl->p2p_blocking == 2) {         /* the link to the next device carries one transfer at a time */
                    int64_t *lf = &link_free[(int64_t)d * pp + (k + 1) % pp];
                    int64_t depart = now > *lf ? now : *lf;
                    arrive = depart + pf[k];
                    *lf = arrive;
                }
                heap_push(h, arrive, EV_ARRIVE_F, k + 1, j, 0);
                mb_[d] += pf[k]; nev++;
            }
            if (kd == 0 && k + 1 == S) sc->arrB[(int64_t)k * m + j] = 1;     /* turn-around on the last virtual stage */
            if (kd == 1 && k > 0) {
                int64_t arrive = now + pb[k];
                if (cl->p2p_blocking == 1) arrive = now;
                if (cl->p2p_blocking == 2) {
                    int64_t *lf = &link_free[(int64_t)d * pp + (k - 1) % pp];
                    int64_t depart = now > *lf ? now : *lf;
                    arrive = depart + pb[k];
                    *lf = arrive;
                }
                heap_push(h, arrive, EV_ARRIVE_B, k - 1, j, 0);
                mb_[d] += pb[k]; nev++;
            }
            if (next[d] == per_dev && dp > 1 && cap == 0) {       /* trailing gradient all-reduce of the device */
                int64_t G = 0;
                for (int c = 0; c < vch; c++)
                    for (int l = bnd[c * pp + d]; l < bnd[c * pp + d + 1]; l++) G += grad[l];
                if (G > 0) {
                    int64_t dd = allreduce_ns(cl, dp, G);
                    heap_push(h, now + dd, EV_AR_DONE, k, 0, 0);
                    mb_[d] += dd;
                    if (tl_ar) { tl_ar[d] = now; tl_ar[pp + d] = now + dd; }
                }
            }
            TRY_START_I(d);
            break;
        }
        case EV_ARRIVE_F:
            sc->arrF[(int64_t)k * m + e.mb] = 1;
            TRY_START_I(d);
            break;
        case EV_ARRIVE_B:
            sc->arrB[(int64_t)k * m + e.mb] = 1;
            TRY_START_I(d);
            break;
        case EV_GRAD_READY: {                        /* bucketed, overlapped gradient all-reduce of device d */
            acc[d] += grad[e.layer];
            pend[d]--;
            while (acc[d] >= cap || (pend[d] == 0 && acc[d] > 0)) {
                int64_t bytes = acc[d] >= cap ? cap : acc[d];
                int64_t dd = allreduce_ns(cl, dp, bytes);
                int64_t st = comm_free[d] > now ? comm_free[d] : now;
                comm_free[d] = st + dd;
                heap_push(h, comm_free[d], EV_AR_DONE, k, 0, 0);
                mb_[d] += dd;
                if (tl_ar) { if (tl_ar[d] < 0) tl_ar[d] = st; tl_ar[pp + d] = comm_free[d]; }
                acc[d] -= bytes;
            }
            break;
        }
        case EV_AR_DONE:
            nev++;
            break;
        }
    }
#undef TRY_START_I
    free(task_vs);
    FREE_I();
#undef FREE_I
    res->batch_ns = now;
    res->num_events = nev;
    for (int d = 0; d < pp; d++) {
        if (comp_busy) comp_busy[d] = cb[d];
        if (comm_busy) comm_busy[d] = mb_[d];
        if (util) util[d] = now > 0 ? (double)cb[d] / (double)now : 0.0;
    }
}

/* ---- explicit schedule (schedule 4) ------------------------------------------------------
 * Algorithm 1 takes the pipeline schedule S as an input: which device runs which stage-task of
 * which micro-batch, in which order (Sec. 4.3).  Here the caller supplies exactly that.  A
 * schedule is a block of 32-bit words:
 *   [0] pp devices  [1] S virtual stages  [2] m micro-batches  [3] nparts: parts of the layer
 *   partition that the stages refer to  [4] replicas (the gradient all-reduce of a device spans
 *   dp * replicas ranks)  [5 .. 5+pp] first task of every device's list and the task total
 *   then S triples (device of the stage, its part, the stage before it in its pipeline or -1)
 *   then the tasks, device after device: kind << 31 | stage << 16 | micro-batch.
 * F(k, j) needs F(prev[k], j) and its p2p event; B(k, j) needs B(next[k], j) and its p2p event,
 * or, on a stage without successor, its own F(k, j).  A device runs its list in order; a task
 * starts when the device is free and its input has arrived.  One gradient all-reduce per device
 * after its list, over the bytes of the parts of all stages it holds.  With a bucket size
 * (extension): the gradients of a stage are complete in the last backward task of that stage on the
 * device's list, layer by layer from the last layer of its part to the first; the device fills its
 * buckets in that order, full buckets are reduced at once and queue on the device's communication
 * stream, what is left after the device's last gradient goes as one more event; a stage without a
 * backward task on the list produces no gradient.  A schedule that cannot be
 * run to its end (an input that never arrives) is invalid, as is any malformed block.  With
 * p2p_blocking == 2 a link is an ordered pair (sending device, receiving device) and carries one
 * transfer at a time.
 * Per-stage outputs are per device. */
static void simulate_explicit(const costs_t *co, const cluster_t *cl,
                              int32_t dp, int32_t tp, int32_t pp, int32_t m,
                              const int32_t *w, int64_t nwords, const uint8_t *bnd_in, int64_t bnd_avail,
                              scratch_t *sc, result_t *res,
                              int64_t *comp_busy, int64_t *comm_busy, double *util,
                              int64_t *tl_start, int64_t *tl_end /* [2][S][m] or NULL; tasks not listed keep what is there */,
                              int64_t *tl_ar /* [2][pp] or NULL */) {
    const int L = co->L;
    res->status = ST_INVALID;
    res->batch_ns = INT64_MAX;
    res->num_events = 0;
    if (dp < 1 || tp < 1 || pp < 1 || pp > MAX_PP || m < 1) return;
    if ((int64_t)dp * tp * pp != cl->num_devices) return;
    if (!w || nwords < 5 + pp + 1) return;
    const int S = w[1], nparts = w[3], replicas = w[4];
    if (w[0] != pp || w[2] != m || S < 1 || nparts < 1 || nparts > L || replicas < 1) return;
    if (bnd_in && bnd_avail < (int64_t)nparts + 1) return;
    const int32_t *dev_off = w + 5;
    const int64_t ntask = dev_off[pp];
    if (dev_off[0] != 0 || ntask < 0 || ntask > 2ll * S * m) return;
    for (int d = 0; d < pp; d++) if (dev_off[d + 1] < dev_off[d]) return;
    if (nwords != 5 + pp + 1 + 3ll * S + ntask) return;           /* bounds S by the block's length */
    const int32_t *st = dev_off + pp + 1, *tasks = st + 3 * (int64_t)S;
    int v = -1;
    for (int i = 0; i < co->V; i++) if (co->variant_tp[i] == tp) { v = i; break; }
    if (v < 0) return;
    /* by virtual stage: device, part, the stage before and after it in its pipeline, outgoing p2p events */
    int *place = (int *)malloc((size_t)S * 4 * sizeof(int)), *part = place + S, *prev = part + S, *next = prev + S;
    int64_t *pf = (int64_t *)calloc((size_t)S * 2, sizeof(int64_t)), *pb = pf + S;
    int *bnd = (int *)malloc((size_t)(nparts + 1) * sizeof(int));
    int64_t *link_free = (int64_t *)calloc((size_t)pp * pp, sizeof(int64_t));   /* [sender][receiver]: free again at */
    uint8_t *seen = NULL;
    int64_t *last_bwd = NULL;
#define FREE_X() do { free(place); free(pf); free(bnd); free(link_free); free(seen); free(last_bwd); } while (0)
    for (int k = 0; k < S; k++) next[k] = -1;
    for (int k = 0; k < S; k++) {
        place[k] = st[3 * k]; part[k] = st[3 * k + 1]; prev[k] = st[3 * k + 2];
        if (place[k] < 0 || place[k] >= pp || part[k] < 0 || part[k] >= nparts || prev[k] < -1 || prev[k] >= S || prev[k] == k) {
            FREE_X(); return;
        }
    }
    for (int k = 0; k < S; k++) if (prev[k] >= 0) { if (next[prev[k]] >= 0) { FREE_X(); return; } next[prev[k]] = k; }
    if (bnd_in) {
        int okp = 1;
        for (int q = 0; q <= nparts; q++) bnd[q] = bnd_in[q];
        if (bnd[0] != 0 || bnd[nparts] != L) okp = 0;
        for (int q = 0; q < nparts && okp; q++) if (bnd[q + 1] <= bnd[q]) okp = 0;
        if (!okp) { FREE_X(); return; }
    } else {
        for (int q = 0; q <= nparts; q++) bnd[q] = (int)(((int64_t)q * L) / nparts);
    }
    /* every task once, on the device of its stage */
    int64_t narr = (int64_t)S * m;
    if (narr > sc->cap_arr) {
        sc->cap_arr = narr;
        sc->arrF = (uint8_t *)realloc(sc->arrF, (size_t)narr);
        sc->arrB = (uint8_t *)realloc(sc->arrB, (size_t)narr);
    }
    seen = (uint8_t *)calloc((size_t)(2 * narr), 1);
    int okl = 1;
    for (int d = 0; d < pp && okl; d++)
        for (int64_t i = dev_off[d]; i < dev_off[d + 1]; i++) {
            uint32_t x = (uint32_t)tasks[i];
            int kd = x >> 31, k = (x >> 16) & 0x7fff, j = x & 0xffff;
            if (k >= S || j >= m || place[k] != d || seen[((int64_t)kd * S + k) * m + j]) { okl = 0; break; }
            seen[((int64_t)kd * S + k) * m + j] = 1;
        }
    if (!okl) { FREE_X(); return; }

    const int64_t *fc = co->fc + (int64_t)v * L, *bc = co->bc + (int64_t)v * L;
    const int64_t *fa = co->fa + (int64_t)v * L, *ba = co->ba + (int64_t)v * L;
    const int64_t *act = co->act + (int64_t)v * L, *grad = co->grad + (int64_t)v * L;
    const int64_t *a2a = co->a2a + (int64_t)v * L;
    /* p2p event on the edge prev[k] -> k, both directions: the activation that leaves prev[k] */
    const int64_t g = cl->gpus_per_node;
    for (int k = 0; k < S; k++) if (prev[k] >= 0) {
        int q = prev[k];
        int64_t na = ((int64_t)place[q] * tp * dp) / g, nb = ((int64_t)place[k] * tp * dp) / g;
        int64_t t = p2p_ns(cl, act[bnd[part[q] + 1] - 1], na == nb ? 0 : 1);
        pf[q] = t;          /* sent by the forward task of prev[k] */
        pb[k] = t;          /* sent by the backward task of k */
    }
    {
        unsigned __int128 t1 = 0;
        for (int k = 0; k < S; k++) {
            for (int l = bnd[part[k]]; l < bnd[part[k] + 1]; l++) {
                t1 += (unsigned __int128)(fc[l] + bc[l]);
                if (tp > 1) t1 += (unsigned __int128)(fa[l] + ba[l]);
                t1 += 2 * (unsigned __int128)alltoall_ns(cl, dp, a2a[l]);
            }
            t1 += (unsigned __int128)(pf[k] + pb[k]);
        }
        if (t1 * (unsigned __int128)m >= ((unsigned __int128)1 << 53)) { FREE_X(); res->status = ST_RANGE; return; }
    }

    memset(sc->arrF, 0, (size_t)narr);
    memset(sc->arrB, 0, (size_t)narr);
    uint8_t *doneF = seen;                 /* reused: forward task has ended */
    memset(doneF, 0, (size_t)(2 * narr));
    heap_t *h = &sc->heap;
    h->n = 0; h->seq = 0;
    int64_t nxt[64];
    uint8_t busy[64];
    int64_t cb[64], mb_[64];
    int64_t comm_free[64], acc[64], pend[64];     /* DP communication stream, open bucket bytes, gradients still to come */
    for (int d = 0; d < pp; d++) { nxt[d] = dev_off[d]; busy[d] = 0; cb[d] = 0; mb_[d] = 0; comm_free[d] = 0; acc[d] = 0; pend[d] = 0; }
    int64_t nev = 0, now = 0, ran = 0;
    if (tl_ar) for (int d = 0; d < 2 * pp; d++) tl_ar[d] = -1;
    const int64_t cap = cl->bucket, ranks = (int64_t)dp * replicas;
    /* by stage: the last backward task of the stage on its device's list, -1 = none */
    last_bwd = (int64_t *)malloc((size_t)S * sizeof(int64_t));
    for (int q = 0; q < S; q++) last_bwd[q] = -1;
    for (int64_t i = 0; i < ntask; i++) {
        uint32_t x = (uint32_t)tasks[i];
        if (x >> 31) last_bwd[(x >> 16) & 0x7fff] = i;
    }
    for (int q = 0; q < S; q++) if (last_bwd[q] >= 0) pend[place[q]] += bnd[part[q] + 1] - bnd[part[q]];

#define TRY_START_X(d_) do {                                                            \
        int d__ = (d_);                                                                 \
        if (!busy[d__] && nxt[d__] < dev_off[d__ + 1]) {                                \
            uint32_t x = (uint32_t)tasks[nxt[d__]];                                     \
            int kd = x >> 31, k = (x >> 16) & 0x7fff, j = x & 0xffff;                   \
            int ready = kd == 0 ? (prev[k] < 0 || sc->arrF[(int64_t)k * m + j])         \
                                : (next[k] < 0 ? doneF[(int64_t)k * m + j] : sc->arrB[(int64_t)k * m + j]); \
            if (ready) {                                                                \
                busy[d__] = 1;                                                          \
                int64_t t = now;                                                        \
                if (tl_start) tl_start[((int64_t)kd * S + k) * m + j] = t;              \
                if (kd == 0) {                                                          \
                    for (int l = bnd[part[k]]; l < bnd[part[k] + 1]; l++) {             \
                        t += fc[l]; cb[d__] += fc[l];                                   \
                        if (tp > 1) { t += fa[l]; mb_[d__] += fa[l]; }                  \
                        int64_t y = alltoall_ns(cl, dp, a2a[l]);                        \
                        t += y; mb_[d__] += y;                                          \
                    }                                                                   \
                } else {                                                                \
                    for (int l = bnd[part[k] + 1] - 1; l >= bnd[part[k]]; l--) {        \
                        t += bc[l]; cb[d__] += bc[l];                                   \
                        if (tp > 1) { t += ba[l]; mb_[d__] += ba[l]; }                  \
                        int64_t y = alltoall_ns(cl, dp, a2a[l]);                        \
                        t += y; mb_[d__] += y;                                          \
                        if (nxt[d__] == last_bwd[k] && cap > 0 && ranks > 1)            \
                            heap_push(h, t, EV_GRAD_READY, k, j, l);                    \
                    }                                                                   \
                }                                                                       \
                if (cl->p2p_blocking == 1) {                                            \
                    if (kd == 0 && next[k] >= 0) t += pf[k];                            \
                    if (kd == 1 && prev[k] >= 0) t += pb[k];                            \
                }                                                                       \
                heap_push(h, t, EV_TASK_DONE, k, j, kd);                                \
            }                                                                           \
        }                                                                               \
    } while (0)

    for (int d = 0; d < pp; d++) TRY_START_X(d);
    while (h->n > 0) {
        event_t e = heap_pop(h);
        now = e.t;
        int k = e.stage, d = place[k];
        switch (e.kind) {
        case EV_TASK_DONE: {
            int kd = e.layer, j = e.mb;
            nev++; ran++;
            if (tl_end) tl_end[((int64_t)kd * S + k) * m + j] = now;
            busy[d] = 0;
            nxt[d]++;
            if (kd == 0) {
                doneF[(int64_t)k * m + j] = 1;
                if (next[k] >= 0) {
                    int64_t arrive = now + pf[k];
                    if (cl->p2p_blocking == 1) arrive = now;
                    if (cl->p2p_blocking == 2) {     /* one transfer at a time from this device to that one */
                        int64_t *lf = &link_free[(int64_t)d * pp + place[next[k]]];
                        int64_t depart = now > *lf ? now : *lf;
                        arrive = depart + pf[k];
                        *lf = arrive;
                    }
                    heap_push(h, arrive, EV_ARRIVE_F, next[k], j, 0);
                    mb_[d] += pf[k]; nev++;
                }
            } else if (prev[k] >= 0) {
                int64_t arrive = now + pb[k];
                if (cl->p2p_blocking == 1) arrive = now;
                if (cl->p2p_blocking == 2) {
                    int64_t *lf = &link_free[(int64_t)d * pp + place[prev[k]]];
                    int64_t depart = now > *lf ? now : *lf;
                    arrive = depart + pb[k];
                    *lf = arrive;
                }
                heap_push(h, arrive, EV_ARRIVE_B, prev[k], j, 0);
                mb_[d] += pb[k]; nev++;
            }
            if (nxt[d] == dev_off[d + 1] && ranks > 1 && cap == 0) {      /* the device's gradient all-reduce */
                int64_t G = 0;
                for (int q = 0; q < S; q++) if (place[q] == d)
                    for (int l = bnd[part[q]]; l < bnd[part[q] + 1]; l++) G += grad[l];
                if (G > 0) {
                    int64_t dd = allreduce_ns(cl, (int64_t)dp * replicas, G);
                    heap_push(h, now + dd, EV_AR_DONE, k, 0, 0);
                    mb_[d] += dd;
                    if (tl_ar) { tl_ar[d] = now; tl_ar[pp + d] = now + dd; }
                }
            }
            TRY_START_X(d);
            break;
        }
        case EV_ARRIVE_F:
            sc->arrF[(int64_t)k * m + e.mb] = 1;
            TRY_START_X(d);
            break;
        case EV_ARRIVE_B:
            sc->arrB[(int64_t)k * m + e.mb] = 1;
            TRY_START_X(d);
            break;
        case EV_GRAD_READY: {                        /* bucketed, overlapped gradient all-reduce of device d */
            acc[d] += grad[e.layer];
            pend[d]--;
            while (acc[d] >= cap || (pend[d] == 0 && acc[d] > 0)) {
                int64_t bytes = acc[d] >= cap ? cap : acc[d];
                int64_t dd = allreduce_ns(cl, ranks, bytes);
                int64_t st = comm_free[d] > now ? comm_free[d] : now;
                comm_free[d] = st + dd;
                heap_push(h, comm_free[d], EV_AR_DONE, k, 0, 0);
                mb_[d] += dd;
                if (tl_ar) { if (tl_ar[d] < 0) tl_ar[d] = st; tl_ar[pp + d] = comm_free[d]; }
                acc[d] -= bytes;
            }
            break;
        }
        case EV_AR_DONE:
            nev++;
            break;
        }
    }
#undef TRY_START_X
    FREE_X();
#undef FREE_X
    if (ran != ntask) return;                  /* some list could not be run to its end */
    res->status = ST_OK;
    res->batch_ns = now;
    res->num_events = nev;
    for (int d = 0; d < pp; d++) {
        if (comp_busy) comp_busy[d] = cb[d];
        if (comm_busy) comm_busy[d] = mb_[d];
        if (util) util[d] = now > 0 ? (double)cb[d] / (double)now : 0.0;
    }
}

/* Per-candidate outputs: status, batch_ns, num_events [C]; stage_off [C+1] is written here
 * (exclusive prefix of pp over candidates with status 0); comp/comm/util are ragged
 * arrays indexed stage_off[c] + s and must hold sum(pp) entries. */
int oracle_simulate(int32_t L, int32_t V, const int32_t *variant_tp,
                    const int64_t *fc, const int64_t *bc, const int64_t *fa, const int64_t *ba,
                    const int64_t *act, const int64_t *grad, const int64_t *a2a,
                    int32_t num_devices, int32_t gpus_per_node,
                    const int64_t *alpha2, const int64_t *beta2, int64_t bucket, int32_t p2p_blocking,
                    int64_t C, const int32_t *dp, const int32_t *tp, const int32_t *pp, const int32_t *m,
                    const uint8_t *schedule, const int32_t *chunks /* or NULL */, const int64_t *part_off,
                    const uint8_t *part_pool, int64_t part_pool_len,
                    int64_t n_sched, const int64_t *sched_off /* [n_sched+1] or NULL */, const int32_t *sched_words,
                    int64_t sched_words_len,
                    int32_t *status, int64_t *batch_ns, int64_t *num_events, int64_t *stage_off,
                    int64_t *comp_busy, int64_t *comm_busy, double *util,
                    int64_t *tl_start, int64_t *tl_end, int64_t *tl_ar, int32_t nthreads) {
    if (L < 1 || V < 1 || C < 0 || beta2[0] < 1 || beta2[1] < 1 || gpus_per_node < 1) return -1;
    costs_t co = { L, V, variant_tp, fc, bc, fa, ba, act, grad, a2a };
    cluster_t cl = { num_devices, gpus_per_node, { alpha2[0], alpha2[1] }, { beta2[0], beta2[1] }, bucket, p2p_blocking };

    /* Each candidate is simulated into a temporary of its own; the ragged outputs are
     * packed afterwards, once the prefix of the slot counts is known. */
    int64_t *slots = (int64_t *)calloc((size_t)C + 1, sizeof(int64_t));
    if (nthreads < 1) nthreads = 1;
    int64_t **tmp_c = (int64_t **)calloc((size_t)C, sizeof(int64_t *));
#pragma omp parallel num_threads(nthreads)
    {
        scratch_t sc;
        memset(&sc, 0, sizeof sc);
#pragma omp for schedule(dynamic, 8)
        for (int64_t c = 0; c < C; c++) {
            int p = pp[c];
            int64_t *buf = NULL;
            if (p >= 1 && p <= MAX_PP) buf = (int64_t *)malloc((size_t)p * 3 * sizeof(int64_t));
            result_t r;
            /* part_off: -1 = uniform split, else an offset into the pool; anything else is no strategy */
            const int64_t po = part_off[c];
            const uint8_t *b = po >= 0 && po < part_pool_len ? part_pool + po : NULL;
            const int64_t avail = b ? part_pool_len - po : 0;
            if (po < -1 || (po >= 0 && !b)) {
                status[c] = ST_INVALID; batch_ns[c] = INT64_MAX; num_events[c] = 0; slots[c] = 0;
                free(buf);
                continue;
            }
            if (schedule[c] == 4) {
                const int32_t *blk = NULL;
                int64_t nw = 0;
                if (chunks && sched_off && sched_words && chunks[c] >= 0 && chunks[c] < n_sched &&
                    sched_off[chunks[c]] >= 0 && sched_off[chunks[c] + 1] >= sched_off[chunks[c]] &&
                    sched_off[chunks[c] + 1] <= sched_words_len) {
                    blk = sched_words + sched_off[chunks[c]];
                    nw = sched_off[chunks[c] + 1] - sched_off[chunks[c]];
                }
                simulate_explicit(&co, &cl, dp[c], tp[c], p, m[c], blk, nw, b, avail, &sc, &r,
                                  buf, buf ? buf + p : NULL, buf ? (double *)(buf + 2 * p) : NULL,
                                  C == 1 ? tl_start : NULL, C == 1 ? tl_end : NULL, C == 1 ? tl_ar : NULL);
            } else if (schedule[c] == 3)
                simulate_interleaved(&co, &cl, dp[c], tp[c], p, m[c], chunks ? chunks[c] : 0 /* no chunk counts: invalid */, b, avail, &sc, &r,
                                     buf, buf ? buf + p : NULL, buf ? (double *)(buf + 2 * p) : NULL,
                                     C == 1 ? tl_start : NULL, C == 1 ? tl_end : NULL, C == 1 ? tl_ar : NULL);
            else
                simulate_one(&co, &cl, dp[c], tp[c], p, m[c], schedule[c], b, avail, &sc, &r,
                             buf, buf ? buf + p : NULL, buf ? (double *)(buf + 2 * p) : NULL,
                             C == 1 ? tl_start : NULL, C == 1 ? tl_end : NULL, C == 1 ? tl_ar : NULL);
            status[c] = r.status;
            batch_ns[c] = r.batch_ns;
            num_events[c] = r.num_events;
            slots[c] = r.status == ST_OK ? p : 0;
            if (r.status != ST_OK) { free(buf); buf = NULL; }
            tmp_c[c] = buf;
        }
        free(sc.heap.a); free(sc.task_kind); free(sc.task_mb); free(sc.arrF); free(sc.arrB);
    }
    int64_t off = 0;
    for (int64_t c = 0; c < C; c++) {
        stage_off[c] = off;
        int64_t p = slots[c];
        if (p) {
            memcpy(comp_busy + off, tmp_c[c], (size_t)p * 8);
            memcpy(comm_busy + off, tmp_c[c] + p, (size_t)p * 8);
            if (util) memcpy(util + off, tmp_c[c] + 2 * p, (size_t)p * 8);
            free(tmp_c[c]);
        }
        off += p;
    }
    stage_off[C] = off;
    free(tmp_c);
    free(slots);
    return 0;
}

/* The composed events of every pipeline stage, written out from their definitions with plain loops
 * over the stage's layers (Sec. 4.3: a layer is a computation event, plus an all-reduce event when
 * MP > 1; a stage is the list of its layers' events).  For the candidates with status[c] == 0 and
 * one of the schedules 0..2, entry i = stage_off[c] + s of the columns
 *   0 FC, 2 BC  forward / backward computation of the stage's layers
 *   1 FA, 3 BA  communication inside the stage: the layers' all-reduce events (tp > 1) and
 *               all-to-all events over the dp group
 *   4 PF, 5 PB  p2p event towards stage s+1 / s-1: the activation that crosses that boundary
 *   6 G         gradient bytes, 7 AR the ring all-reduce of G over dp ranks (Sec. 4.2 volume; 0 for
 *               the asynchronous schedule, which has no such event)
 * and layer_lo / layer_hi = the stage's layers [lo, hi).  Candidates of the schedules 3 and 4 keep
 * zeros (their outputs are per device).  tab is [8][n] with n = stage_off[C]. */
int oracle_stage_table(int32_t L, int32_t V, const int32_t *variant_tp,
                       const int64_t *fc, const int64_t *bc, const int64_t *fa, const int64_t *ba,
                       const int64_t *act, const int64_t *grad, const int64_t *a2a,
                       int32_t num_devices, int32_t gpus_per_node,
                       const int64_t *alpha2, const int64_t *beta2,
                       int64_t C, const int32_t *dp, const int32_t *tp, const int32_t *pp,
                       const uint8_t *schedule, const int64_t *part_off, const uint8_t *part_pool,
                       const int32_t *status, const int64_t *stage_off,
                       int64_t *tab, int32_t *layer_lo, int32_t *layer_hi) {
    if (L < 1 || V < 1 || C < 0) return -1;
    cluster_t cl = { num_devices, gpus_per_node, { alpha2[0], alpha2[1] }, { beta2[0], beta2[1] }, 0, 0 };
    const int64_t n = stage_off[C];
    memset(tab, 0, (size_t)(8 * n) * sizeof(int64_t));
    memset(layer_lo, 0, (size_t)n * sizeof(int32_t));
    memset(layer_hi, 0, (size_t)n * sizeof(int32_t));
    for (int64_t c = 0; c < C; c++) {
        if (status[c] != ST_OK || schedule[c] > 2) continue;
        const int P = pp[c];
        int v = -1;
        for (int i = 0; i < V; i++) if (variant_tp[i] == tp[c]) { v = i; break; }
        if (v < 0) return -2;
        for (int s = 0; s < P; s++) {
            const int lo = part_off[c] >= 0 ? part_pool[part_off[c] + s] : (int)(((int64_t)s * L) / P);
            const int hi = part_off[c] >= 0 ? part_pool[part_off[c] + s + 1] : (int)(((int64_t)(s + 1) * L) / P);
            const int64_t i = stage_off[c] + s;
            int64_t FC = 0, FA = 0, BC = 0, BA = 0, G = 0;
            for (int l = lo; l < hi; l++) {
                const int64_t x = (int64_t)v * L + l;
                FC += fc[x];
                BC += bc[x];
                if (tp[c] > 1) { FA += fa[x]; BA += ba[x]; }
                FA += alltoall_ns(&cl, dp[c], a2a[x]);
                BA += alltoall_ns(&cl, dp[c], a2a[x]);
                G += grad[x];
            }
            /* ranks ordered tp fastest, then dp, then pp: node of the first rank of a pipeline position */
            const int64_t per = (int64_t)tp[c] * dp[c], g = gpus_per_node;
            int64_t PF = 0, PB = 0;
            if (s + 1 < P) PF = p2p_ns(&cl, act[(int64_t)v * L + hi - 1], (s * per) / g == ((s + 1) * per) / g ? 0 : 1);
            if (s > 0) PB = p2p_ns(&cl, act[(int64_t)v * L + lo - 1], ((s - 1) * per) / g == (s * per) / g ? 0 : 1);
            tab[0 * n + i] = FC; tab[1 * n + i] = FA; tab[2 * n + i] = BC; tab[3 * n + i] = BA;
            tab[4 * n + i] = PF; tab[5 * n + i] = PB; tab[6 * n + i] = G;
            tab[7 * n + i] = schedule[c] == 2 ? 0 : allreduce_ns(&cl, dp[c], G);
            layer_lo[i] = lo; layer_hi[i] = hi;
        }
    }
    return 0;
}

/* Grid-search step (Sec. 6): index of the best candidate, ties to the lowest index.
 * objective 0: smallest batch_ns.  objective 1: smallest batch_ns / weight (time per sample),
 * compared exactly as batch_a * w_b < batch_b * w_a.  Candidates with batch_ns == INT64_MAX
 * (unreachable) or, for objective 1, weight <= 0 never win.  best = {index or -1, batch_ns}. */
int oracle_search(const int64_t *batch_ns, const int64_t *weight, int64_t C, int32_t objective, int64_t *best) {
    int64_t bi = -1;
    for (int64_t c = 0; c < C; c++) {
        if (batch_ns[c] == INT64_MAX) continue;
        if (objective == 1 && weight[c] <= 0) continue;
        if (bi < 0) { bi = c; continue; }
        int better;
        if (objective == 0) {
            better = batch_ns[c] < batch_ns[bi];
        } else {
            unsigned __int128 l = (unsigned __int128)batch_ns[c] * (unsigned __int128)weight[bi];
            unsigned __int128 r = (unsigned __int128)batch_ns[bi] * (unsigned __int128)weight[c];
            better = l < r;
        }
        if (better) bi = c;
    }
    best[0] = bi;
    best[1] = bi < 0 ? INT64_MAX : batch_ns[bi];
    return 0;
}
