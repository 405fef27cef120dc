// Host-side dispatching: length-aware buffer, student-number controller, dispatcher loop (see sp_dispatch.h for the
// passages of the paper and the readings D1-D8).  Plain C++ on the host; nothing here touches the GPU.
//
// Buffer storage: a ring of `capacity` elements addressed by a sequence number that only grows (element e lives in
// slot e mod capacity; the queue is the range [head, tail)).  The dictionary of the paper is an array indexed by the
// bin (a perfect hash: there are max_len / bin_width bins) that holds the sequence number of the most recently appended
// element of the bin, or -1.  An entry is live exactly when it is >= head, so dispatching the first element needs no
// search: it clears the entry only if the entry is the element's own number (D3).  Samples of an element sit in the
// element's fixed run of max_elem cells, so nothing is allocated after sp_lab_create.
#include <algorithm>
#include <cstdlib>
#include <functional>
#include <new>
#include <queue>
#include <vector>

#include "sp.h"
#include "sp_dispatch.h"

struct sp_lab {
    int32_t bin_width, max_len, max_elem, capacity, nbins;
    int64_t head, tail;            // sequence numbers: queue = [head, tail)
    int64_t nsamples;
    int32_t* ebin;                 // [capacity] bin of the element in a slot
    int32_t* ecount;               // [capacity] samples in it
    int64_t* ids;                  // [capacity][max_elem]
    int32_t* lens;                 // [capacity][max_elem]
    int64_t* where;                // [nbins] sequence number of the last element of the bin, -1 if none was appended
};

struct sp_ctl {
    int32_t total, slots, k_min, k;
    int64_t window_us, empty_since;   // empty_since < 0: the buffer is not known to be empty
};

namespace {

inline int32_t clip_len(const sp_lab* b, int32_t length) { return length < 1 ? 1 : (length > b->max_len ? b->max_len : length); }
inline int32_t bin_of(const sp_lab* b, int32_t length) { return (clip_len(b, length) + b->bin_width - 1) / b->bin_width - 1; }

bool lab_shape_ok(int32_t bin_width, int32_t max_len, int32_t max_elem, int32_t capacity)
{
    return bin_width >= 1 && max_len >= bin_width && max_len % bin_width == 0 && max_elem >= 1 && capacity >= 1;
}

bool ctl_shape_ok(int32_t total, int32_t slots, int32_t k_min, int64_t window_us, int32_t k_start)
{
    return total >= 1 && k_min >= 1 && k_min <= total && slots >= total && window_us >= 0 &&
           (k_start == 0 || (k_start >= k_min && k_start <= total));
}

}  // namespace

extern "C" {

int sp_lab_create(int32_t bin_width, int32_t max_len, int32_t max_elem, int32_t capacity, sp_lab** out)
{
    if (!out) return SP_EINVAL;
    *out = nullptr;
    if (!lab_shape_ok(bin_width, max_len, max_elem, capacity)) return SP_ESHAPE;
    sp_lab* b = new (std::nothrow) sp_lab{};
    if (!b) return SP_ENOMEM;
    b->bin_width = bin_width; b->max_len = max_len; b->max_elem = max_elem; b->capacity = capacity;
    b->nbins = max_len / bin_width;
    b->ebin = (int32_t*)malloc(sizeof(int32_t) * (size_t)capacity);
    b->ecount = (int32_t*)malloc(sizeof(int32_t) * (size_t)capacity);
    b->ids = (int64_t*)malloc(sizeof(int64_t) * (size_t)capacity * (size_t)max_elem);
    b->lens = (int32_t*)malloc(sizeof(int32_t) * (size_t)capacity * (size_t)max_elem);
    b->where = (int64_t*)malloc(sizeof(int64_t) * (size_t)b->nbins);
    if (!b->ebin || !b->ecount || !b->ids || !b->lens || !b->where) { sp_lab_free(b); return SP_ENOMEM; }
    for (int32_t i = 0; i < b->nbins; ++i) b->where[i] = -1;
    *out = b;
    return SP_OK;
}

void sp_lab_free(sp_lab* b)
{
    if (!b) return;
    free(b->ebin); free(b->ecount); free(b->ids); free(b->lens); free(b->where);
    delete b;
}

int sp_lab_bin_of(const sp_lab* b, int32_t length) { return b ? bin_of(b, length) : SP_EINVAL; }

int sp_lab_bin_len(const sp_lab* b, int32_t bin)
{
    if (!b || bin < 0 || bin >= b->nbins) return SP_EINVAL;
    return (bin + 1) * b->bin_width;
}

int sp_lab_push(sp_lab* b, int64_t sample_id, int32_t length, int32_t* joined)
{
    if (!b || !joined) return SP_EINVAL;
    const int32_t bin = bin_of(b, length);
    const int64_t e = b->where[bin];
    if (e >= b->head) {                                   // the bin has an element in the queue (D2: its newest one)
        const int64_t slot = e % b->capacity;
        if (b->ecount[slot] < b->max_elem) {
            const int64_t cell = slot * b->max_elem + b->ecount[slot]++;
            b->ids[cell] = sample_id;
            b->lens[cell] = clip_len(b, length);
            ++b->nsamples;
            *joined = 1;
            return SP_OK;
        }
    }
    if (b->tail - b->head >= b->capacity) return SP_EFULL;   // D4
    const int64_t slot = b->tail % b->capacity;
    b->ebin[slot] = bin;
    b->ecount[slot] = 1;
    b->ids[slot * b->max_elem] = sample_id;
    b->lens[slot * b->max_elem] = clip_len(b, length);
    b->where[bin] = b->tail++;
    ++b->nsamples;
    *joined = 0;
    return SP_OK;
}

int sp_lab_pop(sp_lab* b, int32_t* bin, int32_t* bin_len, int64_t* ids, int32_t* lengths, int32_t* count)
{
    if (!b || !bin || !bin_len || !ids || !lengths || !count) return SP_EINVAL;
    if (b->tail == b->head) return SP_EEMPTY;
    const int64_t slot = b->head % b->capacity;
    const int32_t n = b->ecount[slot];
    for (int32_t i = 0; i < n; ++i) { ids[i] = b->ids[slot * b->max_elem + i]; lengths[i] = b->lens[slot * b->max_elem + i]; }
    *bin = b->ebin[slot];
    *bin_len = (b->ebin[slot] + 1) * b->bin_width;
    *count = n;
    if (b->where[b->ebin[slot]] == b->head) b->where[b->ebin[slot]] = -1;   // D3
    ++b->head;
    b->nsamples -= n;
    return SP_OK;
}

int sp_lab_elements(const sp_lab* b) { return b ? (int)(b->tail - b->head) : SP_EINVAL; }
int sp_lab_samples(const sp_lab* b) { return b ? (int)b->nsamples : SP_EINVAL; }

int sp_ctl_create(int32_t total_students, int32_t slots, int32_t k_min, int64_t window_us, int32_t k_start, sp_ctl** out)
{
    if (!out) return SP_EINVAL;
    *out = nullptr;
    if (!ctl_shape_ok(total_students, slots, k_min, window_us, k_start)) return SP_ESHAPE;
    sp_ctl* c = new (std::nothrow) sp_ctl{};
    if (!c) return SP_ENOMEM;
    c->total = total_students; c->slots = slots; c->k_min = k_min; c->window_us = window_us;
    c->k = k_start ? k_start : total_students;
    c->empty_since = -1;
    *out = c;
    return SP_OK;
}

void sp_ctl_free(sp_ctl* c) { delete c; }
int sp_ctl_k(const sp_ctl* c) { return c ? c->k : SP_EINVAL; }
int sp_ctl_groups(const sp_ctl* c) { return c ? c->slots / c->k : SP_EINVAL; }

int sp_ctl_on_buffered(sp_ctl* c, int32_t buffer_elements)
{
    if (!c) return SP_EINVAL;
    c->empty_since = -1;
    if (buffer_elements >= c->slots / c->k && c->k > c->k_min) { --c->k; return 1; }   // D5
    return 0;
}

int sp_ctl_on_tick(sp_ctl* c, int64_t now_us, int32_t buffer_elements, int32_t busy_groups)
{
    if (!c) return SP_EINVAL;
    if (buffer_elements > 0) { c->empty_since = -1; return 0; }
    if (c->empty_since < 0) c->empty_since = now_us;
    if (now_us - c->empty_since < c->window_us || c->k >= c->total) return 0;
    const int32_t groups = c->slots / c->k;
    const int32_t occupied = busy_groups < groups ? busy_groups : groups;
    if ((int64_t)(groups - occupied) * c->k > occupied) { ++c->k; c->empty_since = now_us; return 1; }   // D6
    return 0;
}

int sp_dispatch_simulate(const sp_sim_config* cfg, const int64_t* arrival_us, const int32_t* lengths, int64_t n,
                         int64_t* dispatch_us, int64_t* done_us, int32_t* k_used, int64_t* element, int64_t* elem_tokens,
                         int32_t* elem_size, int64_t* n_elements, int64_t* trace_us, int32_t* trace_k,
                         int64_t trace_cap, int64_t* n_trace, int64_t* refused)
{
    if (!cfg || !arrival_us || !lengths || !dispatch_us || !done_us || !k_used || !element || !elem_tokens || !elem_size ||
        !n_elements || !n_trace || !refused || !cfg->base_us || !cfg->per_token_ns || (trace_cap > 0 && (!trace_us || !trace_k)))
        return SP_EINVAL;
    if (n < 0 || trace_cap < 0 || !lab_shape_ok(cfg->bin_width, cfg->max_len, cfg->max_elem, cfg->capacity) ||
        !ctl_shape_ok(cfg->total_students, cfg->slots, cfg->k_min, cfg->window_us, cfg->k_start))
        return SP_ESHAPE;
    for (int64_t i = 1; i < n; ++i)
        if (arrival_us[i] < arrival_us[i - 1]) return SP_ESHAPE;

    sp_lab* buf = nullptr;
    sp_ctl* ctl = nullptr;
    int rc = sp_lab_create(cfg->bin_width, cfg->max_len, cfg->max_elem, cfg->capacity, &buf);
    if (rc == SP_OK) rc = sp_ctl_create(cfg->total_students, cfg->slots, cfg->k_min, cfg->window_us, cfg->k_start, &ctl);
    std::vector<int64_t> heap_store, eid;
    std::vector<int32_t> elen;
    try {
        heap_store.reserve((size_t)cfg->slots + 1);
        eid.resize((size_t)cfg->max_elem);
        elen.resize((size_t)cfg->max_elem);
    } catch (const std::bad_alloc&) { rc = rc == SP_OK ? SP_ENOMEM : rc; }
    if (rc != SP_OK) { sp_lab_free(buf); sp_ctl_free(ctl); return rc; }
    // completion times of the busy groups, earliest on top
    std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> running(std::greater<int64_t>(), std::move(heap_store));

    int64_t ne = 0, nt = 0, nref = 0;
    auto note_k = [&](int64_t now) {
        if (nt < trace_cap) { trace_us[nt] = now; trace_k[nt] = ctl->k; }
        ++nt;
    };
    auto dispatch = [&](int64_t now, int32_t bin_len, const int64_t* ids, const int32_t* lens, int32_t count) {
        const int32_t k = ctl->k;
        int64_t tokens = 0;
        if (cfg->padded) tokens = (int64_t)count * bin_len;
        else for (int32_t i = 0; i < count; ++i) tokens += lens[i];
        const int64_t done = now + cfg->base_us[k] + cfg->per_token_ns[k] * tokens / 1000;
        for (int32_t i = 0; i < count; ++i) {
            const int64_t s = ids[i];
            dispatch_us[s] = now; done_us[s] = done; k_used[s] = k; element[s] = ne;
        }
        elem_tokens[ne] = tokens;
        elem_size[ne] = count;
        ++ne;
        running.push(done);
    };
    auto drain = [&](int64_t now) {            // idle groups take buffer elements, first element first
        while (buf->tail != buf->head && (int64_t)running.size() < ctl->slots / ctl->k) {
            int32_t bin, bl, cnt;
            sp_lab_pop(buf, &bin, &bl, eid.data(), elen.data(), &cnt);
            dispatch(now, bl, eid.data(), elen.data(), cnt);
        }
    };

    note_k(0);
    int64_t i = 0;
    while (i < n || !running.empty()) {
        if (!running.empty() && (i >= n || running.top() <= arrival_us[i])) {      // D8: completions first
            const int64_t now = running.top();
            running.pop();
            drain(now);
            if (sp_ctl_on_tick(ctl, now, (int32_t)(buf->tail - buf->head), (int32_t)running.size()) == 1) note_k(now);
            continue;
        }
        const int64_t now = arrival_us[i];
        if (buf->tail == buf->head && (int64_t)running.size() < ctl->slots / ctl->k) {
            const int64_t id = i;
            const int32_t len = clip_len(buf, lengths[i]);
            dispatch(now, (bin_of(buf, lengths[i]) + 1) * buf->bin_width, &id, &len, 1);
            if (sp_ctl_on_tick(ctl, now, 0, (int32_t)running.size()) == 1) note_k(now);
        } else {
            int32_t joined = 0;
            if (sp_lab_push(buf, i, lengths[i], &joined) == SP_OK) {
                if (sp_ctl_on_buffered(ctl, (int32_t)(buf->tail - buf->head)) == 1) {
                    note_k(now);
                    drain(now);                 // more groups may exist now
                }
            } else {
                dispatch_us[i] = done_us[i] = -1; k_used[i] = 0; element[i] = -1;
                ++nref;
            }
        }
        ++i;
    }
    *n_elements = ne; *n_trace = nt; *refused = nref;
    sp_lab_free(buf);
    sp_ctl_free(ctl);
    return SP_OK;
}

}  // extern "C"
