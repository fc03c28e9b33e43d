// Optional per-kernel timing (HIP events on the launch stream) behind
// quota_profile_begin / quota_profile_collect.  Off by default: a scope then
// costs one predictable branch.  Not thread-safe; meant for the benchmark.
#pragma once
#include <hip/hip_runtime.h>
#include "../../include/quota.h"

struct QuotaProfiler {
    bool on = false;
    int used = 0, cap = 0;
    hipEvent_t *ev = nullptr;        // 2 events per recorded launch
    int *kid = nullptr;
    double *ops = nullptr, *bytes = nullptr;
};
extern QuotaProfiler g_quota_prof;

struct ProfScope {
    hipStream_t st;
    int slot;
    ProfScope(int kernel_id, double ops, double bytes, hipStream_t s) : st(s), slot(-1)
    {
        QuotaProfiler &p = g_quota_prof;
        if (!p.on || p.used >= p.cap) return;
        slot = p.used++;
        p.kid[slot] = kernel_id;
        p.ops[slot] = ops;
        p.bytes[slot] = bytes;
        (void)hipEventRecord(p.ev[2 * slot], st);
    }
    ~ProfScope()
    {
        if (slot >= 0) (void)hipEventRecord(g_quota_prof.ev[2 * slot + 1], st);
    }
};
