// Doubling-budget request scheduler (section 4.2 and the DB algorithm of the appendix): two
// priority queues ordered by O_r = Q_r * L_s, same-service same-phase batches, budget doubling,
// starvation thresholds, and EnoughResource() counted in pages of the unified pool.  Host only.
#include <cmath>
#include <set>
#include <tuple>
#include <unordered_map>
#include <vector>

#include "ukv_internal.h"
#include "ukv_sched.h"

namespace {

struct Req {
    uint64_t id;
    uint32_t service, queue, prompt_len, ctx_len, doublings;
    double arrival, budget, priority;
};

// queue order: smaller priority value first, then earlier arrival, then smaller id
using Key = std::tuple<double, double, uint64_t>;

struct ServiceState {
    ukv_sched_service_t prof;
    uint64_t token_bytes;
    uint32_t queued = 0;      // requests of the service in either queue
    double last_served = 0.0; // starvation clock
};

} // namespace

struct ukv_sched {
    std::vector<ServiceState> svc;
    uint64_t page_bytes = 0;
    uint32_t max_batch = 1;
    std::unordered_map<uint64_t, Req> reqs;
    std::set<Key> queue[2]; // wait_queue, decoding_queue: O(log n) insert, erase and smallest
    // per (service, queue): the same keys, so that the best request of one service is O(log n) too
    std::vector<std::set<Key>> by_service[2];

    static Key key_of(const Req &r) { return Key{r.priority, r.arrival, r.id}; }
    void insert(const Req &r) {
        queue[r.queue].insert(key_of(r));
        by_service[r.queue][r.service].insert(key_of(r));
    }
    void erase(const Req &r) {
        queue[r.queue].erase(key_of(r));
        by_service[r.queue][r.service].erase(key_of(r));
    }
    uint64_t pages(uint32_t service, uint64_t n_tokens) const {
        return (n_tokens * svc[service].token_bytes + page_bytes - 1) / page_bytes;
    }
    uint64_t pages_needed(const Req &r) const {
        if (r.queue == UKV_SCHED_WAIT)
            return pages(r.service, r.prompt_len);
        return pages(r.service, (uint64_t)r.ctx_len + 1) - pages(r.service, r.ctx_len);
    }
};

using ukv::set_error;

extern "C" {

int ukv_sched_create(const ukv_pool_t *pool, const ukv_sched_service_t *services, uint32_t n_services,
                     uint32_t max_batch, ukv_sched_t **out) {
    if (!pool || !services || !out) {
        set_error("null argument");
        return UKV_EINVAL;
    }
    *out = nullptr;
    if (n_services != pool->n_services || max_batch == 0) {
        set_error("n_services must equal the pool's and max_batch must be positive");
        return UKV_EINVAL;
    }
    for (uint32_t s = 0; s < n_services; ++s)
        if (!(services[s].mean_time > 0.0) || !(services[s].std_time >= 0.0) ||
            !(services[s].starvation_threshold >= 0.0) || !std::isfinite(services[s].mean_time) ||
            !std::isfinite(services[s].std_time)) {
            set_error("service profile: mean_time > 0, std_time >= 0, starvation_threshold >= 0");
            return UKV_EINVAL;
        }
    ukv_sched *sc = new (std::nothrow) ukv_sched();
    if (!sc) {
        set_error("host allocation failed");
        return UKV_ENOMEM;
    }
    sc->page_bytes = pool->page_bytes;
    sc->max_batch = max_batch;
    sc->svc.resize(n_services);
    for (uint32_t s = 0; s < n_services; ++s) {
        sc->svc[s].prof = services[s];
        sc->svc[s].token_bytes = pool->classes.c[s].token_bytes;
    }
    for (int q = 0; q < 2; ++q)
        sc->by_service[q].resize(n_services);
    *out = sc;
    return UKV_OK;
}

int ukv_sched_destroy(ukv_sched_t *sc) {
    delete sc;
    return UKV_OK;
}

int ukv_sched_add_request(ukv_sched_t *sc, uint64_t id, uint32_t service, uint32_t prompt_len, double now) {
    if (!sc) {
        set_error("null scheduler");
        return UKV_EINVAL;
    }
    if (service >= sc->svc.size() || prompt_len == 0 || sc->reqs.count(id)) {
        set_error("service out of range, empty prompt, or id already queued");
        return UKV_EINVAL;
    }
    ServiceState &s = sc->svc[service];
    if (s.queued == 0)
        s.last_served = now;
    s.queued++;
    const double q = s.prof.mean_time + s.prof.std_time; // InitBudget
    Req r{id, service, UKV_SCHED_WAIT, prompt_len, 0, 0, now, q, q * s.prof.mean_time};
    sc->reqs.emplace(id, r);
    sc->insert(r);
    return UKV_OK;
}

int ukv_sched_next_batch(ukv_sched_t *sc, double now, uint64_t free_pages, uint64_t *ids_out, uint32_t cap,
                         uint32_t *n_out, uint32_t *service_out, uint32_t *queue_out) {
    if (!sc || !ids_out || !n_out || !service_out || !queue_out) {
        set_error("null argument");
        return UKV_EINVAL;
    }
    if (cap < sc->max_batch) {
        set_error("ids_out must hold max_batch ids");
        return UKV_ENOSPC;
    }
    *n_out = 0;
    *service_out = 0;
    *queue_out = UKV_SCHED_WAIT;
    if (sc->reqs.empty())
        return UKV_OK;
    // the most overdue starved service, if any
    int starved = -1;
    double worst = 0.0;
    for (uint32_t s = 0; s < sc->svc.size(); ++s) {
        if (sc->svc[s].queued == 0)
            continue;
        const double over = now - sc->svc[s].last_served - sc->svc[s].prof.starvation_threshold;
        if (over > 0.0 && (starved < 0 || over > worst)) {
            starved = (int)s;
            worst = over;
        }
    }
    // GetHighestPriorityOrStarvedRequest: walk candidates in order until one fits the free pages.
    // Order: the starved service's requests (both queues merged by key), then everyone by key.
    const Req *first = nullptr, *head = nullptr;
    auto consider = [&](const Key &k) {
        const Req &r = sc->reqs.at(std::get<2>(k));
        if (!head)
            head = &r;
        if (!first && sc->pages_needed(r) <= free_pages)
            first = &r;
    };
    auto merged_walk = [&](const std::set<Key> &a, const std::set<Key> &b, int skip_service) {
        auto ia = a.begin(), ib = b.begin();
        while (!first && (ia != a.end() || ib != b.end())) {
            const bool take_a = ib == b.end() || (ia != a.end() && *ia < *ib);
            const Key &k = take_a ? *ia : *ib;
            if (skip_service < 0 || sc->reqs.at(std::get<2>(k)).service != (uint32_t)skip_service)
                consider(k);
            if (take_a)
                ++ia;
            else
                ++ib;
        }
    };
    if (starved >= 0)
        merged_walk(sc->by_service[0][starved], sc->by_service[1][starved], -1);
    if (!first)
        merged_walk(sc->queue[0], sc->queue[1], starved);
    if (!first) { // nothing fits: report what would have been chosen
        *service_out = head->service;
        *queue_out = head->queue;
        return UKV_OK;
    }
    *service_out = first->service;
    *queue_out = first->queue;
    uint64_t used = sc->pages_needed(*first);
    uint32_t n = 0;
    ids_out[n++] = first->id;
    // the rest of the batch: same service, same queue, in priority order, while EnoughResource()
    for (const Key &k : sc->by_service[first->queue][first->service]) {
        if (std::get<2>(k) == first->id)
            continue;
        const Req &r = sc->reqs.at(std::get<2>(k));
        const uint64_t need = sc->pages_needed(r);
        if (n >= sc->max_batch || used + need > free_pages)
            break;
        ids_out[n++] = r.id;
        used += need;
    }
    *n_out = n;
    return UKV_OK;
}

int ukv_sched_complete(ukv_sched_t *sc, const uint64_t *ids, const uint8_t *finished, uint32_t n, double elapsed,
                       double now) {
    if (!sc || (n && (!ids || !finished))) {
        set_error("null argument");
        return UKV_EINVAL;
    }
    for (uint32_t i = 0; i < n; ++i)
        if (!sc->reqs.count(ids[i])) {
            set_error("unknown request id");
            return UKV_EINVAL;
        }
    int service = -1;
    for (uint32_t i = 0; i < n; ++i) {
        Req &r = sc->reqs.at(ids[i]);
        ServiceState &s = sc->svc[r.service];
        service = (int)r.service;
        sc->erase(r);
        if (r.queue == UKV_SCHED_WAIT) {
            r.queue = UKV_SCHED_DECODING;
            r.ctx_len = r.prompt_len;
        } else {
            r.ctx_len += 1;
        }
        if (finished[i]) {
            s.queued--;
            sc->reqs.erase(ids[i]);
            continue;
        }
        r.budget -= elapsed; // UpdateBudget
        if (r.budget <= 0.0) {
            r.doublings += 1;
            r.budget = (s.prof.mean_time + s.prof.std_time) * std::ldexp(1.0, (int)r.doublings);
        }
        r.priority = r.budget * s.prof.mean_time; // UpdatePriority
        sc->insert(r);
    }
    if (service >= 0)
        sc->svc[service].last_served = now;
    return UKV_OK;
}

int ukv_sched_pages_needed(const ukv_sched_t *sc, uint64_t id, uint64_t *pages_out) {
    if (!sc || !pages_out || !sc->reqs.count(id)) {
        set_error("null argument or unknown request id");
        return UKV_EINVAL;
    }
    *pages_out = sc->pages_needed(sc->reqs.at(id));
    return UKV_OK;
}

int ukv_sched_request_info(const ukv_sched_t *sc, uint64_t id, ukv_sched_request_t *out) {
    if (!sc || !out || !sc->reqs.count(id)) {
        set_error("null argument or unknown request id");
        return UKV_EINVAL;
    }
    const Req &r = sc->reqs.at(id);
    *out = ukv_sched_request_t{r.service, r.queue, r.prompt_len, r.ctx_len, r.doublings, r.arrival, r.budget, r.priority};
    return UKV_OK;
}

uint32_t ukv_sched_pending(const ukv_sched_t *sc) { return sc ? (uint32_t)sc->reqs.size() : 0; }

} // extern "C"
