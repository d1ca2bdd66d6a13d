/*
 * TEST INFRASTRUCTURE -- sequential CPU oracle for the slice-spraying hot path.
 *
 * This file is the checker, not the product.  It is plain, single-threaded C
 * written for legibility against the paper, and shares no code, header, table
 * or helper with the HIP engine.  Only tests, the smoke check and the
 * benchmark's "cpu_baseline" leg may load it.
 *
 * What it follows (TENT, Section 4.2 "Telemetry-Driven Slice Spraying"):
 *   - Slice decomposition: every declared transfer is cut into slices of a
 *     fixed size S; each slice carries its absolute offset inside the transfer
 *     so that it can be written straight to its final place (Section 4.2,
 *     "Slice Decomposition"; the task triple <path, offset, length> of
 *     Algorithm 1).
 *   - Predictive cost: t_d = beta0_d + beta1_d * (A_d + L) / B_d, scaled by the
 *     topology penalty P_d (Eq. 1; Algorithm 1, Stage 2).
 *   - Late binding: each slice goes to the admitted rail with the smallest
 *     predicted completion cost (Section 4.2 opening paragraph); a rail that is
 *     excluded behaves as if its cost were infinite (Section 4.3, "Health
 *     Monitoring"); with no admitted rail the request is deferred (Algorithm 1,
 *     Stage 1).
 *   - Bytes in flight feed back into A_d (Eq. 1's definition of A_d; Section
 *     4.3 "Link-Level Resilience": every issued slice counts in the queue
 *     statistics).
 *   - Staged movement through an intermediate buffer, then a direct write at the
 *     slice's absolute destination offset (Section 4.1 "Autonomous Path
 *     Synthesis"; Section 4.4).
 *
 * Readings where the paper is silent (all integer, no floating point):
 *   c1_d   = floor(1e6 * beta1_q8 * penalty_q8 / bw_MBps)   picoseconds per byte, Q16
 *   c0_d   = (lat_ns * 1000 * penalty_q8) >> 8              picoseconds
 *   cost_d = c0_d + (((A_d + L) * c1_d) >> 16)
 *   a DEGRADED rail (Section 4.3: it keeps half its weight and stays eligible) has both
 *   coefficients doubled, i.e. its predicted cost counts twice;
 *   ties go to the lowest rail index; slices are bound in ascending index order;
 *   a rail's staging region packs its slices in bind order; region bases are the
 *   exclusive sum of the rails' byte totals, each rounded up to 256 bytes.
 */
#include <stdint.h>
#include <string.h>

typedef struct { uint32_t seg; uint32_t len; uint64_t off; } ora_extent;

typedef struct {
    uint32_t bw_MBps;
    uint32_t lat_ns;
    uint64_t queued_bytes;
    uint16_t beta1_q8;
    uint16_t penalty_q8;
    uint8_t  health;      /* 0 healthy, 1 degraded, 2 excluded */
} ora_rail;

enum { ORA_OK = 0, ORA_DEFER = 1, ORA_BAD = -1 };

/* ---- slice decomposition (Section 4.2, "Slice Decomposition") ------------- */

static uint64_t desc_len(const uint32_t *ptr, const ora_extent *ext, uint32_t j)
{
    uint64_t total = 0;
    for (uint32_t e = ptr[j]; e < ptr[j + 1]; ++e) total += ext[e].len;
    return total;
}

/* first[j] = index of descriptor j's first slice; first[D] = total slice count. */
uint64_t ora_count_slices(uint32_t D, const uint32_t *ptr, const ora_extent *ext,
                          uint64_t S, uint64_t *first)
{
    uint64_t n = 0;
    for (uint32_t j = 0; j < D; ++j) {
        first[j] = n;
        uint64_t len = desc_len(ptr, ext, j);
        n += (len + S - 1) / S;
    }
    first[D] = n;
    return n;
}

/* Slice k of descriptor j covers bytes [k*S, min((k+1)*S, len_j)) of the transfer. */
void ora_split(uint32_t D, const uint32_t *ptr, const ora_extent *ext, uint64_t S,
               uint32_t *s_desc, uint64_t *s_off, uint32_t *s_len)
{
    uint64_t i = 0;
    for (uint32_t j = 0; j < D; ++j) {
        uint64_t len = desc_len(ptr, ext, j);
        for (uint64_t off = 0; off < len; off += S, ++i) {
            uint64_t rest = len - off;
            s_desc[i] = j;
            s_off[i]  = off;
            s_len[i]  = (uint32_t)(rest < S ? rest : S);
        }
    }
}

/* ---- rail telemetry -> integer cost coefficients (Eq. 1 with penalty) ------ */

void ora_coeffs(const ora_rail *rails, uint32_t R,
                uint64_t *c0, uint64_t *c1, uint8_t *excluded, uint64_t *A)
{
    for (uint32_t d = 0; d < R; ++d) {
        uint64_t bp = (uint64_t)rails[d].beta1_q8 * rails[d].penalty_q8;
        c1[d] = rails[d].bw_MBps ? (1000000ull * bp) / rails[d].bw_MBps : ~0ull;
        c0[d] = ((uint64_t)rails[d].lat_ns * 1000ull * rails[d].penalty_q8) >> 8;
        if (rails[d].health == 1) {      /* degraded: half weight = twice the cost, still eligible */
            c1[d] *= 2;
            c0[d] *= 2;
        }
        excluded[d] = (rails[d].health == 2);
        A[d] = rails[d].queued_bytes;
    }
}

uint64_t ora_cost(uint64_t c0, uint64_t c1, uint64_t A, uint64_t L)
{
    return c0 + (((A + L) * c1) >> 16);
}

/* ---- late binding (Algorithm 1 Stage 1-2, per-slice earliest completion) ---
 * ids == NULL binds slices 0..n-1; otherwise slices ids[0..n-1] in that order.
 * A[] is read and updated (bytes in flight); T[] receives the per-rail byte
 * totals of this call; slices[] receives the per-rail slice counts. */
static void bind_by_cost(uint64_t n, const uint32_t *ids, const uint32_t *s_len, uint32_t R,
                         const uint64_t *c0, const uint64_t *c1, const uint8_t *excluded,
                         uint64_t *A, uint64_t *T, uint64_t *slices,
                         uint32_t *s_rail, uint64_t *s_stage_off)
{
    for (uint64_t q = 0; q < n; ++q) {
        uint64_t i = ids ? ids[q] : q;
        int best = -1;
        uint64_t best_cost = 0;
        for (uint32_t d = 0; d < R; ++d) {
            if (excluded[d]) continue;
            uint64_t cost = ora_cost(c0[d], c1[d], A[d], s_len[i]);
            if (best < 0 || cost < best_cost) { best = (int)d; best_cost = cost; }
        }
        s_rail[i] = (uint32_t)best;
        s_stage_off[i] = T[best];
        T[best] += s_len[i];
        A[best] += s_len[i];
        slices[best] += 1;
    }
}

int ora_bind(uint64_t n, const uint32_t *ids, const uint32_t *s_len, uint32_t R,
             const uint64_t *c0, const uint64_t *c1, const uint8_t *excluded,
             uint64_t *A, uint64_t *T, uint64_t *slices,
             uint32_t *s_rail, uint64_t *s_stage_off)
{
    int admitted = 0;
    for (uint32_t d = 0; d < R; ++d) {
        T[d] = 0;
        slices[d] = 0;
        if (!excluded[d]) admitted = 1;
    }
    if (!admitted) return ORA_DEFER;
    bind_by_cost(n, ids, s_len, R, c0, c1, excluded, A, T, slices, s_rail, s_stage_off);
    return ORA_OK;
}

/* ---- request-level dispatch (Algorithm 1, Stages 1-3; Section 4.2 "Slice Dispatching" and
 * "Quality of Service") -----------------------------------------------------------------------
 * Algorithm 1 is run once per request (here: per declared transfer), in declaration order.
 *   Stage 1: the admitted rails of the request are the non-excluded rails whose current
 *            priority slot accepts the request's priority.  Reading: priorities 0 LOW, 1 MID,
 *            2 HIGH; in window w rail d sits in slot (w + d) mod 3, where slot 0 accepts HIGH
 *            only, slot 1 HIGH and MID, slot 2 everything.  No admitted rail: the request is
 *            deferred, its slices stay pending.
 *   Stage 2: s_d = predicted cost of one slice on rail d (Eq. 1 times the penalty) with the
 *            queue state A_d at the start of the request; s_min its minimum.
 *   Stage 3, mice (request length < theta): candidates are the admitted rails with
 *            s_d <= s_min + floor(gamma_q8 * s_min / 256); the request goes as a whole to the
 *            candidate picked round robin (a counter that advances with every mice request).
 *            Here L of Eq. 1 is the request length.
 *   Stage 3, elephants: weighted proportional spraying with efficiency weights W_d = 1 / s_d
 *            (L of Eq. 1 = the length of the request's first slice).  Reading: the request's
 *            pending slices are dealt in order, each to the admitted rail with the smallest
 *            (m_d + 1) * max(s_d, 1), m_d = slices of this request already dealt to d, ties to
 *            the lowest rail -- so the shares m_d track W_d to within one slice.
 * Every dealt slice adds its bytes to A_d and to the rail's staging region, in dealing order.
 * first[] (D+1 entries) delimits the requests' slices; done[i] != 0 marks slices that are not
 * pending; mode[j] receives 0 (nothing pending), 1 (mice), 2 (elephant) or 3 (deferred);
 * bound[i] is set for every slice dealt.  Returns ORA_DEFER when every rail is excluded. */
typedef struct { uint64_t theta_bytes; uint32_t gamma_q8; uint32_t window; uint64_t rr_start; } ora_dispatch_params;

int ora_dispatch(uint32_t D, const uint64_t *first, const uint32_t *s_len, const uint8_t *done,
                 const uint64_t *req_len, const uint8_t *priority, uint32_t R,
                 const uint64_t *c0, const uint64_t *c1, const uint8_t *excluded,
                 const ora_dispatch_params *dp,
                 uint64_t *A, uint64_t *T, uint64_t *slices,
                 uint32_t *s_rail, uint64_t *s_stage_off, uint8_t *bound, uint8_t *mode, uint64_t *rr_end)
{
    static const uint8_t slot_needs[3] = { 2, 1, 0 };
    uint64_t rr = dp->rr_start;
    int any = 0;
    for (uint32_t d = 0; d < R; ++d) { T[d] = 0; slices[d] = 0; if (!excluded[d]) any = 1; }
    *rr_end = rr;
    if (!any) return ORA_DEFER;

    for (uint32_t j = 0; j < D; ++j) {
        uint64_t n_pending = 0;
        for (uint64_t i = first[j]; i < first[j + 1]; ++i) n_pending += !done[i];
        mode[j] = 0;
        if (n_pending == 0) continue;

        uint8_t admitted[64];
        uint8_t p = priority ? priority[j] : 2;
        int n_adm = 0;
        for (uint32_t d = 0; d < R; ++d) {
            admitted[d] = !excluded[d] && p >= slot_needs[(dp->window + d) % 3];
            n_adm += admitted[d];
        }
        if (n_adm == 0) { mode[j] = 3; continue; }

        uint64_t s[64], s_min = 0;
        int have = 0;
        if (req_len[j] < dp->theta_bytes) {                       /* mice flow */
            for (uint32_t d = 0; d < R; ++d) {
                if (!admitted[d]) continue;
                s[d] = ora_cost(c0[d], c1[d], A[d], req_len[j]);
                if (!have || s[d] < s_min) { s_min = s[d]; have = 1; }
            }
            uint64_t limit = s_min + ((s_min * dp->gamma_q8) >> 8);
            uint32_t cand[64], n_cand = 0;
            for (uint32_t d = 0; d < R; ++d) if (admitted[d] && s[d] <= limit) cand[n_cand++] = d;
            uint32_t pick = cand[rr % n_cand];
            rr += 1;
            for (uint64_t i = first[j]; i < first[j + 1]; ++i) {
                if (done[i]) continue;
                s_rail[i] = pick; s_stage_off[i] = T[pick]; bound[i] = 1;
                T[pick] += s_len[i]; A[pick] += s_len[i]; slices[pick] += 1;
            }
            mode[j] = 1;
        } else {                                                  /* elephant flow */
            uint64_t m[64];
            uint32_t L0 = s_len[first[j]];
            for (uint32_t d = 0; d < R; ++d) {
                m[d] = 0;
                if (!admitted[d]) continue;
                s[d] = ora_cost(c0[d], c1[d], A[d], L0);
                if (s[d] == 0) s[d] = 1;
            }
            for (uint64_t i = first[j]; i < first[j + 1]; ++i) {
                if (done[i]) continue;
                int best = -1;
                uint64_t best_key = 0;
                for (uint32_t d = 0; d < R; ++d) {
                    if (!admitted[d]) continue;
                    uint64_t key = (m[d] + 1) * s[d];
                    if (best < 0 || key < best_key) { best = (int)d; best_key = key; }
                }
                m[best] += 1;
                s_rail[i] = (uint32_t)best; s_stage_off[i] = T[best]; bound[i] = 1;
                T[best] += s_len[i]; A[best] += s_len[i]; slices[best] += 1;
            }
            mode[j] = 2;
        }
    }
    *rr_end = rr;
    return ORA_OK;
}

/* ---- link-level resilience (Section 4.3, "Link-Level Resilience") -----------
 * A slice whose rail reports a hard error goes back to the pending set with its
 * retry count raised by one (counts saturate at 255).  rail_failed[d] != 0 marks
 * the rails that failed; failed[q] is written for the q-th listed slice and
 * per_rail[d] receives the number of slices that failed on rail d. */
uint64_t ora_fail(uint64_t n, const uint32_t *ids, const uint32_t *s_rail, uint32_t R,
                  const uint8_t *rail_failed, uint8_t *s_retry, uint8_t *failed, uint64_t *per_rail)
{
    uint64_t n_failed = 0;
    for (uint32_t d = 0; d < R; ++d) per_rail[d] = 0;
    for (uint64_t q = 0; q < n; ++q) {
        uint64_t i = ids ? ids[q] : q;
        uint32_t d = s_rail[i];
        failed[q] = 0;
        if (d < R && rail_failed[d]) {
            failed[q] = 1;
            if (s_retry[i] < 255) s_retry[i] += 1;
            per_rail[d] += 1;
            n_failed += 1;
        }
    }
    return n_failed;
}

/* Candidate rails of a retried slice, in rotation order.  Two passes (Section 4.3): HEALTHY
 * rails first; only when there is none, DEGRADED rails, and among those the affinity-matched
 * ones (no topology penalty: penalty_q8 <= 256) before any other reachable rail.  Reading:
 * the first non-empty of the three groups is the candidate set, in ascending rail index.
 * Returns the number of candidates (0: every rail is excluded). */
uint32_t ora_rotation_candidates(const ora_rail *rails, uint32_t R, uint32_t *cand)
{
    uint32_t n = 0;
    for (uint32_t d = 0; d < R; ++d) if (rails[d].health == 0) cand[n++] = d;
    if (n) return n;
    for (uint32_t d = 0; d < R; ++d) if (rails[d].health == 1 && rails[d].penalty_q8 <= 256) cand[n++] = d;
    if (n) return n;
    for (uint32_t d = 0; d < R; ++d) if (rails[d].health == 1) cand[n++] = d;
    return n;
}

/* Plan with retried slices (Section 4.3): retries do not go through the cost model but their
 * bytes count in the queue statistics the cost model reads.  Reading: the retried slices
 * (retry count k > 0) are issued first, in ascending slice index; slice i takes candidate
 * number (i + k) mod |candidates|, so that successive retries of one slice walk round the
 * candidate set and slices that failed together spread over it; then the slices with k = 0
 * are bound by predicted cost with A_d and the staging offsets continuing from there.
 * ids lists the slices to plan (NULL = 0..n-1) in ascending order. */
int ora_plan(uint64_t n, const uint32_t *ids, const uint32_t *s_len, const uint8_t *s_retry,
             const ora_rail *rails, uint32_t R,
             const uint64_t *c0, const uint64_t *c1, const uint8_t *excluded,
             uint64_t *A, uint64_t *T, uint64_t *slices,
             uint32_t *s_rail, uint64_t *s_stage_off)
{
    uint32_t cand[64];
    uint32_t n_cand = ora_rotation_candidates(rails, R, cand);
    for (uint32_t d = 0; d < R; ++d) { T[d] = 0; slices[d] = 0; }
    if (n_cand == 0) return ORA_DEFER;

    for (uint64_t q = 0; q < n; ++q) {                 /* pass over the retried slices */
        uint64_t i = ids ? ids[q] : q;
        if (s_retry[i] == 0) continue;
        uint32_t d = cand[(i + s_retry[i]) % n_cand];
        s_rail[i] = d;
        s_stage_off[i] = T[d];
        T[d] += s_len[i];
        A[d] += s_len[i];
        slices[d] += 1;
    }
    for (uint64_t q = 0; q < n; ++q) {                 /* everything else: by predicted cost */
        uint64_t i = ids ? ids[q] : q;
        if (s_retry[i] != 0) continue;
        uint32_t one = (uint32_t)i;
        bind_by_cost(1, &one, s_len, R, c0, c1, excluded, A, T, slices, s_rail, s_stage_off);
    }
    return ORA_OK;
}

/* ---- rail health monitor (Section 4.3, "Health Monitoring") ------------------
 * Three states per rail: HEALTHY (0), DEGRADED (1: half weight, still eligible), PAUSED (2:
 * excluded while a cooldown runs).  The paper gives the states and the rules in words; the
 * reading below fixes them per measurement window, all integers:
 *   - error score of a window = 2 * hard errors + congestion errors, accumulated over
 *     consecutive windows that saw errors (a window without errors clears it); the rail is
 *     paused when the score exceeds 2 * err_threshold, i.e. hard errors beyond the threshold
 *     or congestion errors beyond twice the threshold;
 *   - a pause lasts cooldown_next windows and cooldown_next doubles with every pause; the rail
 *     then re-enters as DEGRADED (gradual re-admission);
 *   - any error below the pause level, or a degradation event, makes the rail DEGRADED; a
 *     window is a degradation event when even its cleanest sample is slow: the bandwidth probe
 *     of the window (Eq. 2; 0 = no sample) is below degrade_q8/256 of the estimate the planner
 *     held before the window;
 *   - a DEGRADED rail is promoted to HEALTHY after recover_windows consecutive windows without
 *     errors and degradation events; promotion resets cooldown_next to cooldown_windows.
 * Errors and events reported for a PAUSED rail are ignored (it carries no traffic). */
typedef struct { uint32_t err_threshold; uint32_t recover_windows; uint32_t cooldown_windows; uint32_t degrade_q8; } ora_monitor_params;
typedef struct { uint32_t state; uint32_t score; uint32_t clean; uint32_t cooldown_left; uint32_t cooldown_next; } ora_monitor;

void ora_monitor_init(uint32_t R, const ora_monitor_params *mp, ora_monitor *mon)
{
    for (uint32_t d = 0; d < R; ++d) {
        mon[d].state = 0; mon[d].score = 0; mon[d].clean = 0;
        mon[d].cooldown_left = 0; mon[d].cooldown_next = mp->cooldown_windows;
    }
}

void ora_monitor_step(uint32_t R, const ora_monitor_params *mp, ora_monitor *mon,
                      const uint32_t *hard, const uint32_t *congestion,
                      const uint32_t *probe_MBps, const uint32_t *bw_MBps)
{
    for (uint32_t d = 0; d < R; ++d) {
        ora_monitor *m = &mon[d];
        if (m->state == 2) {
            if (m->cooldown_left > 0) m->cooldown_left -= 1;
            if (m->cooldown_left == 0) { m->state = 1; m->clean = 0; m->score = 0; }
            continue;
        }
        uint64_t errors = 2ull * hard[d] + congestion[d];
        int event = probe_MBps[d] != 0 && (uint64_t)probe_MBps[d] * 256 < (uint64_t)mp->degrade_q8 * bw_MBps[d];
        if (errors == 0) m->score = 0;
        else m->score = (uint32_t)(m->score + errors > 0xFFFFFFFFull ? 0xFFFFFFFFull : m->score + errors);
        if ((uint64_t)m->score > 2ull * mp->err_threshold) {
            m->state = 2;
            m->score = 0;
            m->clean = 0;
            m->cooldown_left = m->cooldown_next;
            m->cooldown_next = m->cooldown_next >= (1u << 30) ? (1u << 31) : m->cooldown_next * 2;
            if (m->cooldown_left == 0) { m->state = 1; }      /* a zero-length cooldown pauses nothing */
        } else if (errors > 0 || event) {
            m->state = 1;
            m->clean = 0;
        } else if (m->state == 1) {
            m->clean += 1;
            if (m->clean >= mp->recover_windows) { m->state = 0; m->clean = 0; m->cooldown_next = mp->cooldown_windows; }
        }
    }
}

/* Staging region of rail d starts where the regions of rails < d end (256-byte aligned). */
void ora_stage_bases(const uint64_t *T, uint32_t R, uint64_t *base)
{
    uint64_t at = 0;
    for (uint32_t d = 0; d < R; ++d) {
        base[d] = at;
        at += (T[d] + 255) / 256 * 256;
    }
}

/* ---- staged movement (Section 4.1 staging hop; Section 4.4 direct-to-offset) */

/* Copy bytes [off, off+len) of the byte string formed by concatenating the
 * extents ext[lo..hi) between that string and a flat buffer.  to_flat != 0:
 * extents -> flat; otherwise flat -> extents. */
static void move_range(uint8_t *const *seg_base, const ora_extent *ext, uint32_t lo, uint32_t hi,
                       uint64_t off, uint64_t len, uint8_t *flat, int to_flat)
{
    uint64_t pos = 0;                    /* logical position of ext[e]'s first byte */
    for (uint32_t e = lo; e < hi && len > 0; ++e) {
        uint64_t end = pos + ext[e].len;
        if (off < end) {
            uint64_t within = off - pos;
            uint64_t n = end - off;
            if (n > len) n = len;
            uint8_t *paged = seg_base[ext[e].seg] + ext[e].off + within;
            if (to_flat) memcpy(flat, paged, n); else memcpy(paged, flat, n);
            flat += n; off += n; len -= n;
        }
        pos = end;
    }
}

/* Pass 1: every listed slice is gathered from its paged source into its rail's
 * staging region.  Pass 2: every listed slice is written from staging to its
 * absolute offset in the destination.  ids == NULL means slices 0..n-1. */
void ora_execute(uint64_t n, const uint32_t *ids,
                 const uint32_t *s_desc, const uint64_t *s_off, const uint32_t *s_len,
                 const uint32_t *s_rail, const uint64_t *s_stage_off, const uint64_t *rail_base,
                 const uint32_t *src_ptr, const ora_extent *src_ext,
                 const uint32_t *dst_ptr, const ora_extent *dst_ext,
                 uint8_t *const *seg_base, uint8_t *staging)
{
    for (uint64_t q = 0; q < n; ++q) {
        uint64_t i = ids ? ids[q] : q;
        uint32_t j = s_desc[i];
        uint8_t *st = staging + rail_base[s_rail[i]] + s_stage_off[i];
        move_range(seg_base, src_ext, src_ptr[j], src_ptr[j + 1], s_off[i], s_len[i], st, 1);
    }
    for (uint64_t q = 0; q < n; ++q) {
        uint64_t i = ids ? ids[q] : q;
        uint32_t j = s_desc[i];
        uint8_t *st = staging + rail_base[s_rail[i]] + s_stage_off[i];
        move_range(seg_base, dst_ext, dst_ptr[j], dst_ptr[j + 1], s_off[i], s_len[i], st, 0);
    }
}

/* ---- bounded, pipelined staging (Section 4.1: the payload is partitioned into pipelined chunks
 * that pass through an intermediate buffer of fixed size) -----------------------------------
 * Reading: the payload is the transfers' logical bytes laid end to end in declaration order
 * (slice i starts at payload position P_i = sum of the lengths of all slices before it);
 * chunk c is the payload range [c * chunk_bytes, (c+1) * chunk_bytes).  Chunks pass through
 * the staging buffer one after the other: all listed (moved) bytes of the chunk are gathered
 * into the buffer, then written from the buffer to their destination.  Inside the buffer every
 * rail still owns one contiguous region per chunk: the chunk's bytes on rail d occupy an interval
 * [lo_d, hi_d) of rail d's staging region (offsets grow with the slice index), they are placed
 * at region_base_d + (offset - lo_d), and region_base_d is the exclusive sum over rails of
 * (hi_d - lo_d) rounded up to 256 bytes.
 * With slots > 1 the buffer is divided into that many slots of slot_bytes each and chunk c uses
 * slot c mod slots, so that a chunk can be filled while its predecessor is still being drained
 * (the overlap of consecutive stages described in Section 4.1); the bytes that end up in every
 * slot do not depend on how the stages overlap in time.
 * Returns 0, or -1 when some chunk needs more than a slot or the slots exceed the buffer (nothing is
 * moved then). */
int ora_execute_bounded(uint64_t n_all, uint64_t n, const uint32_t *ids,
                        const uint32_t *s_desc, const uint64_t *s_off,
                        const uint32_t *s_rail, const uint64_t *s_stage_off, uint32_t R,
                        const uint32_t *src_ptr, const ora_extent *src_ext,
                        const uint32_t *dst_ptr, const ora_extent *dst_ext,
                        uint8_t *const *seg_base, uint8_t *staging, uint64_t staging_cap,
                        uint64_t chunk_bytes, uint32_t slots, uint64_t slot_bytes,
                        const uint64_t *P /* n_all + 1 payload positions */)
{
    if (slots == 0 || slot_bytes > staging_cap / slots) return -1;
    uint64_t payload = P[n_all];
    uint64_t n_chunks = (payload + chunk_bytes - 1) / chunk_bytes;
    for (int pass = 0; pass < 2; ++pass) {            /* pass 0 only checks the capacity */
        uint64_t q_first = 0;
        for (uint64_t c = 0; c < n_chunks; ++c) {
            uint64_t c_lo = c * chunk_bytes, c_hi = c_lo + chunk_bytes;
            uint64_t lo[64], hi[64], base[64];
            for (uint32_t d = 0; d < R; ++d) { lo[d] = ~0ull; hi[d] = 0; }
            while (q_first < n && P[(ids ? ids[q_first] : q_first) + 1] <= c_lo) ++q_first;
            for (uint64_t q = q_first; q < n; ++q) {
                uint64_t i = ids ? ids[q] : q;
                if (P[i] >= c_hi) break;
                uint64_t from = P[i] > c_lo ? P[i] : c_lo, to = P[i + 1] < c_hi ? P[i + 1] : c_hi;
                uint64_t reg = s_stage_off[i] + (from - P[i]);
                uint32_t d = s_rail[i];
                if (reg < lo[d]) lo[d] = reg;
                if (reg + (to - from) > hi[d]) hi[d] = reg + (to - from);
            }
            uint64_t at = 0;
            for (uint32_t d = 0; d < R; ++d) {
                base[d] = at;
                if (hi[d] > lo[d] && lo[d] != ~0ull) at += (hi[d] - lo[d] + 255) / 256 * 256;
            }
            if (at > slot_bytes) return -1;
            if (pass == 0) continue;
            for (int to_dst = 0; to_dst < 2; ++to_dst)
                for (uint64_t q = q_first; q < n; ++q) {
                    uint64_t i = ids ? ids[q] : q;
                    if (P[i] >= c_hi) break;
                    uint64_t from = P[i] > c_lo ? P[i] : c_lo, to = P[i + 1] < c_hi ? P[i + 1] : c_hi;
                    uint64_t x = from - P[i];
                    uint32_t d = s_rail[i], j = s_desc[i];
                    uint8_t *st = staging + (c % slots) * slot_bytes + base[d] + (s_stage_off[i] + x - lo[d]);
                    if (!to_dst) move_range(seg_base, src_ext, src_ptr[j], src_ptr[j + 1], s_off[i] + x, to - from, st, 1);
                    else         move_range(seg_base, dst_ext, dst_ptr[j], dst_ptr[j + 1], s_off[i] + x, to - from, st, 0);
                }
        }
    }
    return 0;
}

/* ---- rail simulator for the re-planning workload ---------------------------
 * A rail drains its queue in order: the bytes that were already queued
 * (queued[d]) go first, then this plan's slices in staging order.  A slice
 * completes in the epoch iff its last byte fits the rail's byte budget;
 * everything else returns to the pending set and is re-planned (Section 4.3,
 * idempotent retry).  done[q] is written for the q-th listed slice. */
uint64_t ora_retire(uint64_t n, const uint32_t *ids, const uint32_t *s_len,
                    const uint32_t *s_rail, const uint64_t *s_stage_off,
                    const uint64_t *queued, const uint64_t *budget, uint8_t *done)
{
    uint64_t n_done = 0;
    for (uint64_t q = 0; q < n; ++q) {
        uint64_t i = ids ? ids[q] : q;
        uint32_t d = s_rail[i];
        uint64_t last = queued[d] + s_stage_off[i] + s_len[i];
        int fits = last >= queued[d] /* no wrap */ && last <= budget[d];
        done[q] = (uint8_t)fits;
        n_done += (uint64_t)fits;
    }
    return n_done;
}

/* ---- telemetry feedback (Section 4.2: Eq. 2 "peak picking" and the smoothing filter) --------
 * Eq. 2: within a measurement window the bandwidth probe of rail d is
 *     B_probe_d = min{ B_hw_d, max_i alpha * L_i / (tau_i - delta) }
 * over the slices i that completed on d in the window (L_i bytes, tau_i end-to-end latency), and
 * the estimate B_d follows the probes through an exponentially weighted moving average.
 * Integer reading: tau and delta in ns, bandwidths in 1e6 B/s, so a sample is
 *     floor(alpha_q8 * L * 1000 / (256 * (tau - delta)))        (alpha in Q8.8)
 * a slice with tau <= delta counts as a sample at the hardware bandwidth; the update is
 *     B_d <- max(1, (ewma_q8 * B_probe_d + (256 - ewma_q8) * B_d) >> 8)
 * and a rail without a completed slice in the window keeps its estimate. */
typedef struct { uint32_t hw_MBps; uint32_t alpha_q8; uint32_t delta_ns; uint32_t ewma_q8; } ora_probe_params;

/* Rail simulator: latency of a slice = the rail's fixed latency plus the time the rail needs, at
 * its true bandwidth, to drain the bytes queued before the plan, the slices staged ahead of this
 * one and the slice itself.  ceil(x * 1000 / bw) is taken as (x / bw) * 1000 + ceil((x % bw) * 1000 / bw). */
void ora_sim_latency(uint64_t n, const uint32_t *ids, const uint32_t *s_len, const uint32_t *s_rail,
                     const uint64_t *s_stage_off, const uint64_t *queued, const uint32_t *lat_ns,
                     const uint32_t *true_bw_MBps, uint64_t *tau_ns)
{
    for (uint64_t q = 0; q < n; ++q) {
        uint64_t i = ids ? ids[q] : q;
        uint32_t d = s_rail[i];
        uint64_t x = queued[d] + s_stage_off[i] + s_len[i];
        uint64_t bw = true_bw_MBps[d];
        uint64_t whole = x / bw, rest = x % bw;
        tau_ns[i] = lat_ns[d] + whole * 1000 + (rest * 1000 + bw - 1) / bw;
    }
}

void ora_probe(uint64_t n, const uint32_t *ids, const uint32_t *s_len, const uint32_t *s_rail,
               const uint64_t *tau_ns, uint32_t R, const ora_probe_params *pp,
               uint32_t *bw_MBps /* in: estimate, out: updated estimate */,
               uint32_t *probe_MBps /* out: B_probe, 0 where no slice completed */)
{
    uint64_t peak[64];
    uint8_t seen[64];
    for (uint32_t d = 0; d < R; ++d) { peak[d] = 0; seen[d] = 0; }
    for (uint64_t q = 0; q < n; ++q) {
        uint64_t i = ids ? ids[q] : q;
        uint32_t d = s_rail[i];
        uint64_t sample;
        if (tau_ns[i] <= pp[d].delta_ns) {
            sample = pp[d].hw_MBps;
        } else {
            uint64_t t = tau_ns[i] - pp[d].delta_ns;
            sample = ((uint64_t)pp[d].alpha_q8 * s_len[i] * 1000) / (256 * t);
        }
        if (sample > peak[d]) peak[d] = sample;
        seen[d] = 1;
    }
    for (uint32_t d = 0; d < R; ++d) {
        probe_MBps[d] = 0;
        if (!seen[d]) continue;
        uint64_t probe = peak[d] < pp[d].hw_MBps ? peak[d] : pp[d].hw_MBps;
        uint64_t next = ((uint64_t)pp[d].ewma_q8 * probe + (uint64_t)(256 - pp[d].ewma_q8) * bw_MBps[d]) >> 8;
        probe_MBps[d] = (uint32_t)probe;
        bw_MBps[d] = (uint32_t)(next ? next : 1);
    }
}
