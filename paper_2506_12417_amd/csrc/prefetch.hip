// Asynchronous expert fetching by overwrite (section 4.3): pinned-host -> device-slot copies on
// a stream of the engine's own, ordered against the compute stream with two events per slot:
//   ready[s]  recorded on the copy stream after the copy into slot s; the compute stream waits
//             on it before the expert's FFN (read-after-write)
//   freed[s]  recorded on the compute stream after the last use of slot s; the copy stream
//             waits on it before overwriting the slot (write-after-read)
// Nothing is written back to the host: the finished expert is simply overwritten.
#include "common.h"
#include <vector>
#include <new>

struct moe_prefetch {
    int n_slots;
    size_t slot_bytes;
    char* base;
    hipStream_t copy_stream;
    std::vector<hipEvent_t> ready, freed;
    std::vector<int> expert;        // expert held by each slot, -1 = never used
    std::vector<char> released;     // slot's expert has been released
    std::vector<long long> release_seq;
    long long seq;
};

extern "C" int moe_prefetch_create(moe_prefetch** h, int n_slots, size_t slot_bytes, void* slot_base) {
    MOE_REQUIRE(h && slot_base, MOE_ERR_ARG, "moe_prefetch_create: null pointer");
    MOE_REQUIRE(n_slots >= 1 && n_slots <= 4096 && slot_bytes >= 1, MOE_ERR_ARG, "moe_prefetch_create: n_slots=%d slot_bytes=%zu", n_slots, slot_bytes);
    moe_prefetch* p = new (std::nothrow) moe_prefetch();
    MOE_REQUIRE(p, MOE_ERR_ARG, "moe_prefetch_create: out of host memory");
    p->n_slots = n_slots;
    p->slot_bytes = slot_bytes;
    p->base = (char*)slot_base;
    p->seq = 0;
    p->copy_stream = nullptr;
    hipError_t e = hipStreamCreateWithFlags(&p->copy_stream, hipStreamNonBlocking);
    if (e != hipSuccess) { delete p; return moe_fail(MOE_ERR_HIP, "moe_prefetch_create: stream: %s", hipGetErrorString(e)); }
    p->ready.assign(n_slots, nullptr);
    p->freed.assign(n_slots, nullptr);
    p->expert.assign(n_slots, -1);
    p->released.assign(n_slots, 0);
    p->release_seq.assign(n_slots, 0);
    for (int s = 0; s < n_slots; ++s) {
        hipError_t e1 = hipEventCreateWithFlags(&p->ready[s], hipEventDisableTiming);
        hipError_t e2 = hipEventCreateWithFlags(&p->freed[s], hipEventDisableTiming);
        if (e1 != hipSuccess || e2 != hipSuccess) {
            moe_prefetch_destroy(p);
            return moe_fail(MOE_ERR_HIP, "moe_prefetch_create: event creation failed");
        }
    }
    *h = p;
    return MOE_OK;
}

static int find_slot(const moe_prefetch* p, int expert_id) {
    for (int s = 0; s < p->n_slots; ++s)
        if (p->expert[s] == expert_id) return s;
    return -1;
}

extern "C" int moe_prefetch_experts(moe_prefetch* h, const int32_t* expert_ids, int n, const void* const* host_w,
                                    size_t bytes_each, const void** slot_ptrs_out) {
    MOE_REQUIRE(h && (n == 0 || (expert_ids && host_w)), MOE_ERR_ARG, "moe_prefetch_experts: null pointer");
    MOE_REQUIRE(n >= 0, MOE_ERR_ARG, "moe_prefetch_experts: n=%d", n);
    MOE_REQUIRE(bytes_each >= 1 && bytes_each <= h->slot_bytes, MOE_ERR_CAPACITY, "moe_prefetch_experts: %zu bytes do not fit a slot of %zu", bytes_each, h->slot_bytes);
    // choose every slot first, so that an error leaves nothing enqueued
    std::vector<int> slot(n, -1);
    std::vector<int> exp_after(h->expert);
    std::vector<char> rel_after(h->released);
    for (int i = 0; i < n; ++i) {
        MOE_REQUIRE(expert_ids[i] >= 0, MOE_ERR_ARG, "moe_prefetch_experts: expert id %d", expert_ids[i]);
        MOE_REQUIRE(host_w[i], MOE_ERR_ARG, "moe_prefetch_experts: null host pointer for expert %d", expert_ids[i]);
        for (int s = 0; s < h->n_slots; ++s)
            MOE_REQUIRE(!(exp_after[s] == expert_ids[i] && !rel_after[s]), MOE_ERR_ARG, "moe_prefetch_experts: expert %d is already resident", expert_ids[i]);
        int pick = -1;
        for (int s = 0; s < h->n_slots && pick < 0; ++s)
            if (exp_after[s] < 0) pick = s;                     // a slot never used
        if (pick < 0) {
            long long best = 0;
            for (int s = 0; s < h->n_slots; ++s)
                if (rel_after[s] && (pick < 0 || h->release_seq[s] < best)) { pick = s; best = h->release_seq[s]; }
        }
        MOE_REQUIRE(pick >= 0, MOE_ERR_CAPACITY, "moe_prefetch_experts: no free slot for expert %d (%d slots, none released)", expert_ids[i], h->n_slots);
        slot[i] = pick;
        exp_after[pick] = expert_ids[i];
        rel_after[pick] = 0;
    }
    for (int i = 0; i < n; ++i) {
        const int s = slot[i];
        if (h->expert[s] >= 0)   // overwrite: wait until the previous expert's last use is done
            MOE_CHECK_HIP(hipStreamWaitEvent(h->copy_stream, h->freed[s], 0));
        MOE_CHECK_HIP(hipMemcpyAsync(h->base + (size_t)s * h->slot_bytes, host_w[i], bytes_each, hipMemcpyHostToDevice, h->copy_stream));
        MOE_CHECK_HIP(hipEventRecord(h->ready[s], h->copy_stream));
        h->expert[s] = expert_ids[i];
        h->released[s] = 0;
        if (slot_ptrs_out) slot_ptrs_out[i] = h->base + (size_t)s * h->slot_bytes;
    }
    return MOE_OK;
}

extern "C" int moe_prefetch_wait(moe_prefetch* h, int expert_id, void* stream) {
    MOE_REQUIRE(h, MOE_ERR_ARG, "moe_prefetch_wait: null handle");
    const int s = find_slot(h, expert_id);
    MOE_REQUIRE(s >= 0, MOE_ERR_ARG, "moe_prefetch_wait: expert %d is in no slot", expert_id);
    MOE_CHECK_HIP(hipStreamWaitEvent((hipStream_t)stream, h->ready[s], 0));
    return MOE_OK;
}

extern "C" int moe_prefetch_release(moe_prefetch* h, int expert_id, void* stream) {
    MOE_REQUIRE(h, MOE_ERR_ARG, "moe_prefetch_release: null handle");
    const int s = find_slot(h, expert_id);
    MOE_REQUIRE(s >= 0 && !h->released[s], MOE_ERR_ARG, "moe_prefetch_release: expert %d is not resident", expert_id);
    MOE_CHECK_HIP(hipEventRecord(h->freed[s], (hipStream_t)stream));
    h->released[s] = 1;
    h->release_seq[s] = ++h->seq;
    return MOE_OK;
}

extern "C" int moe_prefetch_reset(moe_prefetch* h) {
    MOE_REQUIRE(h, MOE_ERR_ARG, "moe_prefetch_reset: null handle");
    for (int s = 0; s < h->n_slots; ++s)
        MOE_REQUIRE(h->expert[s] < 0 || h->released[s], MOE_ERR_ARG, "moe_prefetch_reset: expert %d has not been released", h->expert[s]);
    // every slot counts as released in slot order: the next fetches take slots 0, 1, 2, ...; a
    // slot that held an expert keeps its "freed" event, so its overwrite still waits for the last use
    for (int s = 0; s < h->n_slots; ++s) {
        if (h->expert[s] >= 0) h->expert[s] = INT32_MAX;      // no expert id matches any more
        h->release_seq[s] = s + 1;
    }
    h->seq = h->n_slots;
    return MOE_OK;
}

extern "C" int moe_prefetch_destroy(moe_prefetch* h) {
    if (!h) return MOE_OK;
    if (h->copy_stream) (void)hipStreamSynchronize(h->copy_stream);
    for (hipEvent_t e : h->ready) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : h->freed) if (e) (void)hipEventDestroy(e);
    if (h->copy_stream) (void)hipStreamDestroy(h->copy_stream);
    delete h;
    return MOE_OK;
}

// ------------------------------------------------------------------------------------------
// moe_set_expert_pointers: the slots that moe_prefetch_experts chose, written into the device
// pointer tables that moe_grouped_ffn reads -- by a tiny kernel on the compute stream, its values
// passed as kernel arguments.  (A host-to-device copy of the table would queue behind the expert
// copies on the same DMA engine and hold the compute stream for the length of a whole expert.)
namespace {
constexpr int SETP_MAX = 16;
struct SetPointersArgs {
    int32_t id[SETP_MAX];
    const void* ptr[SETP_MAX];
};
__global__ void set_pointers_kernel(const void** w_in, const void** w_out, SetPointersArgs a, size_t out_offset, int n) {
    const int i = threadIdx.x;
    if (i < n) {
        w_in[a.id[i]] = a.ptr[i];
        if (w_out) w_out[a.id[i]] = (const char*)a.ptr[i] + out_offset;
    }
}
}  // namespace

extern "C" int moe_set_expert_pointers(const void** w_in, const void** w_out, int E, const int32_t* expert_ids, int n,
                                       const void* const* ptrs, size_t out_offset, void* stream) {
    MOE_REQUIRE(n >= 0 && E >= 1, MOE_ERR_ARG, "moe_set_expert_pointers: n=%d E=%d", n, E);
    if (n == 0) return MOE_OK;
    MOE_REQUIRE(w_in && expert_ids && ptrs, MOE_ERR_ARG, "moe_set_expert_pointers: null pointer");
    for (int i = 0; i < n; ++i) {
        MOE_REQUIRE(expert_ids[i] >= 0 && expert_ids[i] < E, MOE_ERR_ARG, "moe_set_expert_pointers: expert id %d outside [0, %d)", expert_ids[i], E);
        MOE_REQUIRE(ptrs[i], MOE_ERR_ARG, "moe_set_expert_pointers: null pointer for expert %d", expert_ids[i]);
    }
    for (int at = 0; at < n; at += SETP_MAX) {
        SetPointersArgs a;
        const int m = n - at < SETP_MAX ? n - at : SETP_MAX;
        for (int i = 0; i < SETP_MAX; ++i) {
            a.id[i] = i < m ? expert_ids[at + i] : 0;
            a.ptr[i] = i < m ? ptrs[at + i] : nullptr;
        }
        hipLaunchKernelGGL(set_pointers_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, w_in, w_out, a, out_offset, m);
        MOE_CHECK_LAUNCH("moe_set_expert_pointers");
    }
    return MOE_OK;
}
