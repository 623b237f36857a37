// Greedy value-density residency policy: which artifacts to pre-load where (paper section 4.1, equation 1) and
// which to take off the GPU when memory is needed (section 4.3, equations 6 and 7).  Host code only.
//
// Both decisions work on "objects": an artifact, or all BACKBONE artifacts that name the same share_id (one set of
// tensors, placed and sized once, worth the sum of its functions' values -- the shared backbone of section 4.4).
// Value density of an object = value / bytes.  The greedy is the one the paper states: candidates in order of
// density, each taken when capacity and the precedence constraints allow, rescanning after every placement
// (O(n^2) in the number of candidates).
#include <math.h>

#include <algorithm>
#include <map>
#include <utility>
#include <vector>

#include "../../include/lora_sched.h"

namespace {

constexpr int kContainerBit = 1, kGpuBit = 2;

struct Object {
    std::vector<int32_t> members;  // artifact indices
    int32_t kind = 0;
    int32_t first = 0;  // lowest artifact index: the tie-breaker
    double bytes = 0.0, value = 0.0;
    double density() const { return value / bytes; }
};

struct Model {
    std::vector<Object> objects;
    std::vector<int32_t> object_of;              // artifact -> object
    std::vector<std::vector<int32_t>> by_kind;  // per compressed function: artifact index of each kind or -1
    std::vector<int32_t> fn_of;                 // artifact -> compressed function
};

bool finite_nonneg(double v) { return v == v && v >= 0.0 && v < HUGE_VAL; }

// Groups the artifacts into objects and indexes them by function; false on malformed input.
bool build_model(const lora_artifact *arts, int32_t n, Model *m) {
    std::map<int32_t, int32_t> fn_index, share_index;
    m->object_of.assign((size_t)n, -1);
    m->fn_of.assign((size_t)n, -1);
    for (int32_t i = 0; i < n; ++i) {
        const lora_artifact &a = arts[i];
        if (a.kind < LORA_ART_LIBRARY || a.kind > LORA_ART_KERNEL || !finite_nonneg(a.bytes) || !(a.bytes > 0.0) || !finite_nonneg(a.value))
            return false;
        auto fit = fn_index.find(a.function);
        if (fit == fn_index.end()) {
            fit = fn_index.emplace(a.function, (int32_t)m->by_kind.size()).first;
            m->by_kind.push_back(std::vector<int32_t>(4, -1));
        }
        m->fn_of[i] = fit->second;
        int32_t &slot = m->by_kind[(size_t)fit->second][(size_t)a.kind];
        if (slot >= 0) return false;  // one artifact per kind and function
        slot = i;
        if (a.kind == LORA_ART_BACKBONE) {
            auto sit = share_index.find(a.share_id);
            if (sit != share_index.end()) {
                Object &o = m->objects[(size_t)sit->second];
                if (o.bytes != a.bytes) return false;  // one set of tensors has one size
                o.members.push_back(i);
                o.value += a.value;
                m->object_of[i] = sit->second;
                continue;
            }
            share_index.emplace(a.share_id, (int32_t)m->objects.size());
        }
        Object o;
        o.members.push_back(i);
        o.kind = a.kind;
        o.first = i;
        o.bytes = a.bytes;
        o.value = a.value;
        m->object_of[i] = (int32_t)m->objects.size();
        m->objects.push_back(o);
    }
    return true;
}

inline bool place_allowed(int32_t kind, int bit) {
    if (kind == LORA_ART_LIBRARY) return bit == kContainerBit;
    if (kind == LORA_ART_KERNEL) return bit == kGpuBit;
    return true;
}

// Is artifact `dep` of a function (or -1 = the function has none: no requirement) placed with `bit`?
inline bool dep_placed(const Model &m, const std::vector<uint8_t> &placed, int32_t dep, int bit) {
    return dep < 0 || (placed[(size_t)m.object_of[(size_t)dep]] & bit) != 0;
}

// Precedence and coupling constraints of section 4.1 for putting object k into the place `bit`.
bool precedence_ok(const Model &m, const std::vector<uint8_t> &placed, int32_t k, int bit) {
    const Object &o = m.objects[(size_t)k];
    if (o.kind == LORA_ART_BACKBONE || o.kind == LORA_ART_ADAPTER) {  // models need a library in the container first
        bool lib = false;
        for (int32_t a : o.members) lib = lib || dep_placed(m, placed, m.by_kind[(size_t)m.fn_of[(size_t)a]][LORA_ART_LIBRARY], kContainerBit);
        if (!lib) return false;
    }
    const std::vector<int32_t> &mine = m.by_kind[(size_t)m.fn_of[(size_t)o.members[0]]];
    if (o.kind == LORA_ART_ADAPTER && bit == kGpuBit && !dep_placed(m, placed, mine[LORA_ART_BACKBONE], kGpuBit)) return false;
    if (o.kind == LORA_ART_KERNEL &&
        (!dep_placed(m, placed, mine[LORA_ART_BACKBONE], kGpuBit) || !dep_placed(m, placed, mine[LORA_ART_ADAPTER], kGpuBit)))
        return false;
    return true;
}

}  // namespace

extern "C" {

int lora_preload_greedy(const lora_artifact *artifacts, int32_t n, double container_bytes, double gpu_bytes, uint8_t *place_out,
                        double *value_out) {
    if (n < 0 || (n > 0 && (!artifacts || !place_out)) || !finite_nonneg(container_bytes) || !finite_nonneg(gpu_bytes))
        return LORA_SCHED_ERR_INVALID_ARG;
    Model m;
    if (!build_model(artifacts, n, &m)) return LORA_SCHED_ERR_INVALID_ARG;
    struct Cand {
        int32_t obj;
        int bit;
    };
    std::vector<Cand> cands;
    for (int32_t k = 0; k < (int32_t)m.objects.size(); ++k)
        for (int bit : {kContainerBit, kGpuBit})
            if (place_allowed(m.objects[(size_t)k].kind, bit)) cands.push_back(Cand{k, bit});
    std::sort(cands.begin(), cands.end(), [&](const Cand &x, const Cand &y) {
        const double dx = m.objects[(size_t)x.obj].density(), dy = m.objects[(size_t)y.obj].density();
        if (dx != dy) return dx > dy;
        if (m.objects[(size_t)x.obj].first != m.objects[(size_t)y.obj].first) return m.objects[(size_t)x.obj].first < m.objects[(size_t)y.obj].first;
        return x.bit < y.bit;
    });
    std::vector<uint8_t> placed(m.objects.size(), 0);
    double used_container = 0.0, used_gpu = 0.0, value = 0.0;
    // "Place the first candidate in density order that fits, then scan again from the top" -- without the rescans: a
    // candidate that failed on capacity fails for good (capacity only shrinks), so after a placement only the
    // candidates passed over for PRECEDENCE can have become placeable; they are kept in order in `waiting`.
    auto try_place = [&](const Cand &c) -> int {  // 1 placed, 0 no room / already there, -1 precedence not met yet
        const Object &o = m.objects[(size_t)c.obj];
        if (placed[(size_t)c.obj] & c.bit) return 0;
        double &used = c.bit == kContainerBit ? used_container : used_gpu;
        const double cap = c.bit == kContainerBit ? container_bytes : gpu_bytes;
        if (used + o.bytes > cap) return 0;
        if (!precedence_ok(m, placed, c.obj, c.bit)) return -1;
        placed[(size_t)c.obj] |= (uint8_t)c.bit;
        used += o.bytes;
        value += o.value;
        return 1;
    };
    std::vector<size_t> waiting;  // indices into cands, increasing
    auto drain_waiting = [&]() {  // place waiting candidates, densest first, until none of them can go
        for (bool again = true; again;) {
            again = false;
            for (size_t w = 0; w < waiting.size(); ++w) {
                const int r = try_place(cands[waiting[w]]);
                if (r == -1) continue;
                waiting.erase(waiting.begin() + (long)w);  // placed, or out of room for good
                if (r == 1) {
                    again = true;
                    break;
                }
                --w;
            }
        }
    };
    for (size_t i = 0; i < cands.size(); ++i) {
        const int r = try_place(cands[i]);
        if (r == -1) waiting.push_back(i);
        if (r == 1) drain_waiting();
    }
    for (int32_t i = 0; i < n; ++i) place_out[i] = placed[(size_t)m.object_of[(size_t)i]];
    if (value_out) *value_out = value;
    return LORA_SCHED_OK;
}

int lora_offload_greedy(const lora_artifact *artifacts, int32_t n, const uint8_t *on_gpu, double need_bytes, uint8_t *evict_out,
                        double *freed_out, double *value_lost_out) {
    if (n < 0 || (n > 0 && (!artifacts || !on_gpu || !evict_out)) || !(need_bytes == need_bytes) || need_bytes >= HUGE_VAL)
        return LORA_SCHED_ERR_INVALID_ARG;
    Model m;
    if (!build_model(artifacts, n, &m)) return LORA_SCHED_ERR_INVALID_ARG;
    const size_t no = m.objects.size();
    std::vector<uint8_t> here(no, 0), pinned(no, 0), chosen(no, 0);
    for (int32_t i = 0; i < n; ++i) {
        const size_t k = (size_t)m.object_of[(size_t)i];
        if (on_gpu[i] && artifacts[i].kind != LORA_ART_LIBRARY) here[k] = 1;
        if (artifacts[i].pinned) pinned[k] = 1;
    }
    // dependents[k]: objects on the GPU that need object k there (kernels need their models, adapters their backbone)
    std::vector<std::vector<int32_t>> dependents(no);
    for (const std::vector<int32_t> &kinds : m.by_kind) {
        const int32_t bb = kinds[LORA_ART_BACKBONE], ad = kinds[LORA_ART_ADAPTER], ke = kinds[LORA_ART_KERNEL];
        auto obj = [&](int32_t a) { return m.object_of[(size_t)a]; };
        if (bb >= 0) {
            if (ad >= 0 && here[(size_t)obj(ad)]) dependents[(size_t)obj(bb)].push_back(obj(ad));
            if (ke >= 0 && here[(size_t)obj(ke)]) dependents[(size_t)obj(bb)].push_back(obj(ke));
        }
        if (ad >= 0 && ke >= 0 && here[(size_t)obj(ke)]) dependents[(size_t)obj(ad)].push_back(obj(ke));
    }
    double freed = 0.0, lost = 0.0;
    while (freed < need_bytes) {
        int32_t best = -1;
        for (int32_t k = 0; k < (int32_t)no; ++k) {
            if (!here[(size_t)k] || pinned[(size_t)k] || chosen[(size_t)k]) continue;
            bool free_of_dependents = true;
            for (int32_t d : dependents[(size_t)k]) free_of_dependents = free_of_dependents && chosen[(size_t)d];
            if (!free_of_dependents) continue;
            if (best < 0) {
                best = k;
                continue;
            }
            const double dk = m.objects[(size_t)k].density(), db = m.objects[(size_t)best].density();
            if (dk < db || (dk == db && m.objects[(size_t)k].first > m.objects[(size_t)best].first)) best = k;
        }
        if (best < 0) break;
        chosen[(size_t)best] = 1;
        freed += m.objects[(size_t)best].bytes;
        lost += m.objects[(size_t)best].value;
    }
    for (int32_t i = 0; i < n; ++i) evict_out[i] = (uint8_t)(chosen[(size_t)m.object_of[(size_t)i]] && on_gpu[i] ? 1 : 0);
    if (freed_out) *freed_out = freed;
    if (value_lost_out) *value_lost_out = lost;
    return freed >= need_bytes ? LORA_SCHED_OK : LORA_SCHED_ERR_CAPACITY;
}

}  // extern "C"
