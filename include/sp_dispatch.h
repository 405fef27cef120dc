/* Host-side dispatching of Student Parallelism: the length-aware buffer, the student-number controller and the
 * dispatcher loop that joins them.  Plain C ABI; everything except sp_serve_replay (last entry) runs on the host alone
 * (no device memory, no HIP call) and produces the two run-time inputs of sp_forward: a packed batch of samples and
 * k_active.
 *
 * Conventions
 *   - return value 0 (SP_OK) on success, a negative code otherwise (the SP_E* codes of sp.h plus SP_EFULL and
 *     SP_EEMPTY below); no exception, no abort;
 *   - all pointers are host pointers owned by the caller; objects are created once and allocate nothing afterwards:
 *     every operation is O(1) (the paper's claim for the buffer), the loop is O(1) per event;
 *   - times are integer microseconds;
 *   - objects are not thread-safe: one dispatcher thread owns them (the paper's master process).
 *
 * Where the paper is silent the following readings are taken:
 *   D1  a sample of n tokens belongs to bin ceil(n / bin_width) - 1 and is padded to bin_width * ceil(n / bin_width)
 *       tokens; n > max_len is clipped to max_len, n < 1 counts as 1;
 *   D2  the dictionary holds, per bin, the most recently appended element of that bin; a new sample can only join
 *       that element;
 *   D3  dispatching the first element deletes the dictionary entry of its bin only if the entry still points at it;
 *   D4  the storage has a fixed capacity of its own (elements); a push that needs one element more is refused with
 *       SP_EFULL (back-pressure).  The paper's "maximum buffer size", the number of student groups, is the
 *       controller's threshold, not a storage limit;
 *   D5  "the buffer reaches the threshold" is evaluated each time a sample has been buffered; one student is dropped
 *       per such sample, never below k_min;
 *   D6  the buffer-empty window restarts whenever the buffer is non-empty and after every increase;
 *   D7  groups(k) = floor(slots / k), slots = student instances that run concurrently;
 *   D8  events of the same microsecond: completions first, then arrivals in input order;
 *   D9  an element in flight counts as one occupied group whatever student number it was dispatched with: after a
 *       decrease, a new element is admitted while fewer than floor(slots / k_now) elements run, although the older
 *       ones still hold k_old students each until they finish (the paper says the groups "release" their tail
 *       students at once; the service times of the loop in virtual time are optimistic by that much during the
 *       transition).
 */
#ifndef SP_DISPATCH_H
#define SP_DISPATCH_H

#include <stdint.h>

#include "sp.h"

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SP_EFULL = -6,  /* the buffer's storage holds `capacity` elements and the sample cannot join one */
    SP_EEMPTY = -7  /* pop from an empty buffer */
};

/* ---- length-aware buffer (Section 3.3.2 "Inference Sample Dispatching" and its figure; appendix "Details about Sample
 * Dispatching based on Length-aware Buffer"): a first-in-first-out queue of elements, each a small batch of at most
 * max_elem samples of one length bin, and a dictionary from length bin to queue position through which a new sample
 * joins the element of its bin in O(1). ---- */
typedef struct sp_lab sp_lab;

/* bin_width 8, max_len 128, max_elem 4 are the paper's values.  max_len must be a multiple of bin_width; capacity is
 * the number of elements the storage holds (D4).  Errors: SP_EINVAL (null out), SP_ESHAPE (a value < 1, max_len not a
 * multiple of bin_width), SP_ENOMEM. */
int sp_lab_create(int32_t bin_width, int32_t max_len, int32_t max_elem, int32_t capacity, sp_lab** out);
void sp_lab_free(sp_lab* buf);

/* Bin of a sample of `length` tokens (D1), and the padded length of a bin.  A null buffer gives SP_EINVAL. */
int sp_lab_bin_of(const sp_lab* buf, int32_t length);
int sp_lab_bin_len(const sp_lab* buf, int32_t bin);

/* A new sample arrives.  *joined = 1 if it joined the element of its bin, 0 if it became a new last element.
 * Errors: SP_EINVAL, SP_EFULL (nothing changed). */
int sp_lab_push(sp_lab* buf, int64_t sample_id, int32_t length, int32_t* joined);

/* The first element leaves.  ids / lengths: room for max_elem entries; lengths are the clipped sample lengths in
 * arrival order; *bin_len is what the paper's padded batch pads them to.  Errors: SP_EINVAL, SP_EEMPTY. */
int sp_lab_pop(sp_lab* buf, int32_t* bin, int32_t* bin_len, int64_t* ids, int32_t* lengths, int32_t* count);

int sp_lab_elements(const sp_lab* buf);   /* elements queued (what the controller compares with the number of groups) */
int sp_lab_samples(const sp_lab* buf);    /* samples queued */

/* ---- student-number controller (Section 3.3.1; appendix "Details about Student Allocation" and "Student Number
 * Adaptation"): keeps k, the number of active students per group, between k_min and total_students. ---- */
typedef struct sp_ctl sp_ctl;

/* k starts at k_start (0: total_students).  Errors: SP_EINVAL, SP_ESHAPE (k_min, k_start outside 1..total_students,
 * slots < total_students, window_us < 0), SP_ENOMEM. */
int sp_ctl_create(int32_t total_students, int32_t slots, int32_t k_min, int64_t window_us, int32_t k_start,
                  sp_ctl** out);
void sp_ctl_free(sp_ctl* ctl);
int sp_ctl_k(const sp_ctl* ctl);        /* current k_active */
int sp_ctl_groups(const sp_ctl* ctl);   /* groups that k allows (D7) */

/* A sample has just been buffered and the buffer now holds buffer_elements elements (D5).  Returns 1 if a student was
 * dropped, 0 if not, SP_EINVAL for a null controller. */
int sp_ctl_on_buffered(sp_ctl* ctl, int32_t buffer_elements);
/* Any other observation at time now_us (a completion, a direct dispatch).  Returns 1 if a student was added (the
 * buffer has been empty for the window and idle_groups * k > occupied groups, D6), else 0. */
int sp_ctl_on_tick(sp_ctl* ctl, int64_t now_us, int32_t buffer_elements, int32_t busy_groups);

/* ---- the dispatcher loop in virtual time (appendix, the online inference procedure): a sample goes out at once if a
 * group is idle and nothing is buffered, otherwise it is buffered; whenever a group becomes idle the first buffer
 * element goes out.  The service time of an element is base_us[k] + per_token_ns[k] * tokens / 1000 (integer
 * arithmetic), tokens = size * bin length if padded, else the sum of its samples' clipped lengths (fully packed). ---- */
typedef struct sp_sim_config {
    int32_t total_students, slots, k_min, k_start; /* k_start 0: total_students */
    int64_t window_us;
    int32_t bin_width, max_len, max_elem, capacity;
    int32_t padded;                                /* 0: packed tokens, 1: padded to the bin */
    const int64_t* base_us;                        /* [total_students + 1], entry 0 unused */
    const int64_t* per_token_ns;                   /* [total_students + 1] */
} sp_sim_config;

/* arrival_us [n] non-decreasing, lengths [n].  Outputs per sample [n]: dispatch_us, done_us, k_used, element (index of
 * the dispatched element; -1 and times -1 for a refused sample); per dispatched element [n]: elem_tokens, elem_size,
 * *n_elements; the changes of k: trace_us / trace_k [trace_cap] (first entry: time 0, starting k), *n_trace (counts
 * every change, also those beyond trace_cap); *refused.  Errors: SP_EINVAL, SP_ESHAPE (as the constructors; arrivals
 * decreasing), SP_ENOMEM. */
int sp_dispatch_simulate(const sp_sim_config* cfg, const int64_t* arrival_us, const int32_t* lengths, int64_t n,
                         int64_t* dispatch_us, int64_t* done_us, int32_t* k_used, int64_t* element, int64_t* elem_tokens,
                         int32_t* elem_size, int64_t* n_elements, int64_t* trace_us, int32_t* trace_k,
                         int64_t trace_cap, int64_t* n_trace, int64_t* refused);

/* ---- the same loop in real time, on the GPU: replays a list of arrivals against a loaded student group.  The
 * calling thread is the dispatcher (the paper's master process: buffer, controller, dispatching); every student group
 * is a worker thread of the library with its own HIP stream, pinned staging buffers, device inputs / outputs and
 * workspace, which runs one element at a time: ids and offsets to the device, sp_forward with the k_active in force at
 * dispatch, logits back, stream synchronisation.  A sample's latency done_us - arrival_us therefore includes both
 * PCIe copies.  slots / k_min worker threads are started; slots / k of them take work while k students are active.
 * Unlike sp_forward this call allocates (once, before the replay starts: device buffers of slots / k_min groups for
 * max_elem * max_len tokens each) and blocks until the last sample is done.
 * The HIP runtime maps a process's streams onto GPU_MAX_HW_QUEUES hardware queues (default 4; read once, at the
 * process's first HIP call): groups that share a queue serialise their launches, so a process that serves more than
 * four groups should start with that variable set to the number of groups (8 measured well, 16 worse). ---- */
typedef struct sp_serve_config {
    int32_t slots, k_min, k_start;  /* total_students is the loaded group's K; k_start 0: K */
    int64_t window_us;
    int32_t bin_width, max_len, max_elem, capacity;   /* max_len <= the students' max_pos */
    int32_t padded;  /* 1: every sample of an element is padded with pad_id to the bin length (the paper's small batch;
                        the padded tokens are attended to, so only the timing of this variant is meaningful) */
    int32_t pad_id;
} sp_serve_config;

/* model: a group loaded with sp_load_students.  arrival_us [n] non-decreasing, relative to the start of the call;
 * token_ids host [id_offsets[n]], sample i owns [id_offsets[i], id_offsets[i+1]) (its length; only the first max_len
 * tokens are used).  Outputs [n]: dispatch_us, done_us (microseconds since the start of the call), k_used, element
 * (index of the dispatched element, -1 if the sample was refused), logits host float32 [n][classes]; elem_size [n]
 * (first *n_elements entries); *refused; *k_final.
 * Errors: SP_EINVAL, SP_ESHAPE, SP_ENOMEM, SP_EHIP (a HIP call or a forward failed, or no group finished for 10 s). */
int sp_serve_replay(const sp_model* model, const sp_serve_config* cfg, const int64_t* arrival_us,
                    const int32_t* token_ids, const int64_t* id_offsets, int64_t n, int64_t* dispatch_us,
                    int64_t* done_us, int32_t* k_used, int64_t* element, int32_t* elem_size, int64_t* n_elements,
                    float* logits, int64_t* refused, int32_t* k_final);

#ifdef __cplusplus
}
#endif
#endif
