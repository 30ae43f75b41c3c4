// Adapter slot manager: N adapters live in pinned host memory, at most M of them in device
// slots at stable addresses; a batch's adapters are made resident before its apply calls.
//
// This is the serving-side memory scheme of the paper's paged setting (Sec. 4: 512 adapters
// with 32 on the GPU; App. E.2: the active set on the GPU, the catalogue in host memory) and of
// its weight synchronisation for on-policy RL (App. D.4: parameters at stable addresses are
// overwritten in place, so the next launch or graph replay sees the new weights).  Host code
// and asynchronous copies only; see include/preft.h for the contract.
#include "../../include/preft.h"

#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

struct preft_slots {
    int32_t n_adapters = 0, n_slots = 0, n_parts = 0;
    std::vector<size_t> part_bytes, part_offset;   // offsets inside one adapter's record
    size_t record_bytes = 0;                       // one adapter, all parts, parts 256-byte aligned
    char *host_store = nullptr;                    // pinned, n_adapters records
    char *device_slab = nullptr;                   // n_slots records
    void **device_tables = nullptr;                // device: n_parts tables of n_slots pointers
    std::vector<int32_t> slot_of;                  // per adapter: slot or -1
    std::vector<int32_t> adapter_in;               // per slot: adapter or -1
    std::vector<int64_t> last_use;                 // per slot: tick of the last acquire that named it
    std::vector<int64_t> stored;                   // per adapter: bit p set once part p was stored (PREFT_MAX_PARTS <= 64)
    std::vector<hipEvent_t> read_done;             // per adapter: recorded after the latest copy that reads its pinned
                                                   // record (created on first use; null: no copy ever read it)
    int64_t tick = 0, hits = 0, misses = 0, evictions = 0, bytes_copied = 0;
};

namespace {

constexpr size_t PART_ALIGN = 256;

// Marks the point on `st` after which the adapter's pinned record is no longer being read by a copy.
// preft_slots_store waits for it before it overwrites the record, whichever stream the copy ran on
// and whether or not the adapter is still resident.
int mark_record_read(preft_slots *m, int32_t adapter, hipStream_t st)
{
    hipEvent_t &ev = m->read_done[(size_t)adapter];
    if (!ev && hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) { ev = nullptr; return PREFT_EHIP; }
    return hipEventRecord(ev, st) == hipSuccess ? PREFT_OK : PREFT_EHIP;
}

int copy_record(preft_slots *m, int32_t adapter, int32_t slot, hipStream_t st)
{
    if (m->n_parts == 0) return PREFT_OK;
    const char *src = m->host_store + (size_t)adapter * m->record_bytes;
    char *dst = m->device_slab + (size_t)slot * m->record_bytes;
    if (hipMemcpyAsync(dst, src, m->record_bytes, hipMemcpyHostToDevice, st) != hipSuccess) return PREFT_EHIP;
    m->bytes_copied += (int64_t)m->record_bytes;
    return mark_record_read(m, adapter, st);
}

}  // namespace

extern "C" {

int preft_slots_create(preft_slots_t **out, int32_t n_adapters, int32_t n_slots, int32_t n_parts,
                       const size_t *part_bytes)
{
    if (!out || n_adapters < 1 || n_slots < 1 || n_parts < 0 || n_parts > PREFT_MAX_PARTS || (n_parts > 0 && !part_bytes))
        return PREFT_EINVAL;
    preft_slots *m = new (std::nothrow) preft_slots;
    if (!m) return PREFT_EINVAL;
    m->n_adapters = n_adapters;
    m->n_slots = n_slots < n_adapters ? n_slots : n_adapters;
    m->n_parts = n_parts;
    for (int32_t p = 0; p < n_parts; ++p) {
        if (part_bytes[p] == 0) { delete m; return PREFT_EINVAL; }
        m->part_bytes.push_back(part_bytes[p]);
        m->part_offset.push_back(m->record_bytes);
        m->record_bytes += (part_bytes[p] + PART_ALIGN - 1) / PART_ALIGN * PART_ALIGN;
    }
    m->slot_of.assign((size_t)n_adapters, -1);
    m->adapter_in.assign((size_t)m->n_slots, -1);
    m->last_use.assign((size_t)m->n_slots, 0);
    m->stored.assign((size_t)n_adapters, 0);
    m->read_done.assign((size_t)n_adapters, nullptr);
    if (n_parts > 0) {
        // pinned host memory is allocated as such (registering existing memory is not used)
        if (hipHostMalloc(reinterpret_cast<void **>(&m->host_store), (size_t)n_adapters * m->record_bytes,
                          hipHostMallocDefault) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&m->device_slab), (size_t)m->n_slots * m->record_bytes) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&m->device_tables),
                      (size_t)n_parts * m->n_slots * sizeof(void *)) != hipSuccess) {
            preft_slots_destroy(m);
            return PREFT_EHIP;
        }
        std::memset(m->host_store, 0, (size_t)n_adapters * m->record_bytes);
        std::vector<void *> tables((size_t)n_parts * m->n_slots);
        for (int32_t p = 0; p < n_parts; ++p)
            for (int32_t s = 0; s < m->n_slots; ++s)
                tables[(size_t)p * m->n_slots + s] = m->device_slab + (size_t)s * m->record_bytes + m->part_offset[p];
        if (hipMemcpy(m->device_tables, tables.data(), tables.size() * sizeof(void *), hipMemcpyHostToDevice) !=
            hipSuccess) {
            preft_slots_destroy(m);
            return PREFT_EHIP;
        }
    }
    *out = m;
    return PREFT_OK;
}

int preft_slots_destroy(preft_slots_t *m)
{
    if (!m) return PREFT_OK;
    int rc = PREFT_OK;
    for (hipEvent_t ev : m->read_done)
        if (ev && hipEventDestroy(ev) != hipSuccess) rc = PREFT_EHIP;
    if (m->device_tables && hipFree(m->device_tables) != hipSuccess) rc = PREFT_EHIP;
    if (m->device_slab && hipFree(m->device_slab) != hipSuccess) rc = PREFT_EHIP;
    if (m->host_store && hipHostFree(m->host_store) != hipSuccess) rc = PREFT_EHIP;
    delete m;
    return rc;
}

int preft_slots_store(preft_slots_t *m, int32_t adapter, int32_t part, const void *src, void *stream)
{
    if (!m || !src || adapter < 0 || adapter >= m->n_adapters || part < 0 || part >= m->n_parts) return PREFT_EINVAL;
    char *rec = m->host_store + (size_t)adapter * m->record_bytes + m->part_offset[part];
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int32_t slot = m->slot_of[adapter];
    // The pinned record may still be the source of a copy enqueued earlier -- by an acquire that brought
    // the adapter in (it may have been evicted since) or by an earlier refresh, on any stream: wait for
    // the latest such copy, resident or not, before the record is overwritten.
    if (m->read_done[(size_t)adapter] && hipEventSynchronize(m->read_done[(size_t)adapter]) != hipSuccess) return PREFT_EHIP;
    std::memcpy(rec, src, m->part_bytes[part]);
    m->stored[adapter] |= (int64_t)1 << part;
    if (slot >= 0) {                                   // resident: refresh in place, same address
        char *dst = m->device_slab + (size_t)slot * m->record_bytes + m->part_offset[part];
        if (hipMemcpyAsync(dst, rec, m->part_bytes[part], hipMemcpyHostToDevice, st) != hipSuccess) return PREFT_EHIP;
        m->bytes_copied += (int64_t)m->part_bytes[part];
        return mark_record_read(m, adapter, st);
    }
    return PREFT_OK;
}

int preft_slots_acquire(preft_slots_t *m, const int32_t *adapter_ids, int32_t n, int32_t *slot_ids, void *stream)
{
    if (!m || n < 0 || (n > 0 && (!adapter_ids || !slot_ids))) return PREFT_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int64_t now = ++m->tick;
    // first pass: adapters already resident keep their slot and are protected from eviction
    for (int32_t i = 0; i < n; ++i) {
        const int32_t a = adapter_ids[i];
        if (a < 0 || a >= m->n_adapters) continue;
        const int32_t s = m->slot_of[a];
        if (s >= 0) {
            if (m->last_use[s] != now) ++m->hits;
            m->last_use[s] = now;
        }
    }
    // second pass: bring in the rest, each into the least recently used slot this call has not named
    for (int32_t i = 0; i < n; ++i) {
        const int32_t a = adapter_ids[i];
        if (a < 0 || a >= m->n_adapters) { slot_ids[i] = -1; continue; }     // no adapter
        if (m->slot_of[a] < 0) {
            int32_t victim = -1;
            for (int32_t s = 0; s < m->n_slots; ++s) {
                if (m->last_use[s] == now) continue;
                if (victim < 0 || m->last_use[s] < m->last_use[victim]) victim = s;
            }
            if (victim < 0) {
                // more distinct adapters than slots: report, leaving the manager consistent
                for (int32_t j = i; j < n; ++j) slot_ids[j] = -1;
                return PREFT_ECAPACITY;
            }
            if (m->adapter_in[victim] >= 0) {
                m->slot_of[m->adapter_in[victim]] = -1;
                ++m->evictions;
            }
            m->adapter_in[victim] = a;
            m->slot_of[a] = victim;
            m->last_use[victim] = now;
            ++m->misses;
            const int rc = copy_record(m, a, victim, st);
            if (rc != PREFT_OK) return rc;
        }
        slot_ids[i] = m->slot_of[a];
    }
    return PREFT_OK;
}

const void *const *preft_slots_pool(preft_slots_t *m, int32_t part)
{
    if (!m || part < 0 || part >= m->n_parts) return nullptr;
    return reinterpret_cast<const void *const *>(m->device_tables + (size_t)part * m->n_slots);
}

int32_t preft_slots_resident(const preft_slots_t *m, int32_t adapter)
{
    if (!m || adapter < 0 || adapter >= m->n_adapters) return -1;
    return m->slot_of[adapter];
}

int preft_slots_stats(const preft_slots_t *m, int64_t *stats)
{
    if (!m || !stats) return PREFT_EINVAL;
    stats[0] = m->hits;
    stats[1] = m->misses;
    stats[2] = m->evictions;
    stats[3] = m->bytes_copied;
    stats[4] = m->n_slots;
    return PREFT_OK;
}

}  // extern "C"
