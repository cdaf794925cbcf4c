// C ABI of the library: argument checking, plan cache, scratch management and
// dispatch to the kernels.  No exception crosses this boundary.
#include "../../include/cs.h"
#include "kernels.hpp"
#include <cmath>
#include <cstdarg>
#include <new>
#include <cstdio>
#include <cstring>
#include <vector>

using namespace csk;

struct PlanEntry {
    cs_op op;
    const float* psi;
    int G, b, rb;
    Plan plan;
};

struct cs_ctx {
    int device;
    hipStream_t stream;
    void* scratch;
    size_t scratch_bytes;
    int lds_limit;
    int union_hint = 0;
    std::vector<PlanEntry> plans;
    // device arrays of plans for calls that serve several operators at once, keyed by the plans' atom
    // buffers (one buffer per plan for the lifetime of the context)
    struct PlanGroup { std::vector<const float*> key; Plan* d_plans; };
    std::vector<PlanGroup> groups;
    char err[512];
};

// Workspace of cs_block_ffn_static: device memory that exists from the moment the library is loaded, one
// copy per GPU.  Host code never uses this name as an address; cs_create looks the device address up once
// per device (hipGetSymbolAddress) and every later use goes through that pointer.
static __device__ __align__(256) unsigned char scratch[CS_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices] = {};          // per device: address of that device's copy of `scratch`

constexpr size_t kDefaultScratch = 64ull << 20;
constexpr int kMaxWeightedRb = 16;

cs_status fail(cs_ctx* c, cs_status st, const char* fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof c->err, fmt, ap);      // fixed buffer: reporting an error allocates nothing
        va_end(ap);
    }
    return st;
}

cs_status hip_fail(cs_ctx* c, hipError_t e, const char* what) {
    return fail(c, CS_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// Runs the body of an entry point; the host containers used by some of them (plan cache, operator lists)
// may throw when host memory runs out, and nothing may leave the library as an exception.
template <class F>
cs_status guarded(cs_ctx* c, F&& body) noexcept {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(c, CS_ENOMEM, "host memory allocation failed");
    } catch (...) {
        return fail(c, CS_EHIP, "unexpected internal error");
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

OpDesc make_desc(const cs_op& op) {
    OpDesc d;
    d.k0 = (uint32_t)(op.seed & 0xFFFFFFFFull);
    d.k1 = (uint32_t)(op.seed >> 32);
    d.stream = op.stream_id;
    d.ens = op.ens;
    d.m = op.m;
    d.n = op.n;
    d.scale = (float)(1.0 / std::sqrt((double)op.m));
    d.nbits = 1;
    while ((1ll << d.nbits) < (long long)op.n) ++d.nbits;
    return d;
}

cs_status check_op(cs_ctx* c, const cs_op* op, const char* who) {
    if (!op) return fail(c, CS_EINVAL, "%s: operator is NULL", who);
    if (op->ens != CS_GAUSS && op->ens != CS_RADEMACHER && op->ens != CS_SRHT)
        return fail(c, CS_EINVAL, "%s: unknown ensemble %d", who, op->ens);
    if (op->m < 1 || op->n < 1) return fail(c, CS_EINVAL, "%s: operator needs m >= 1 and n >= 1 (m=%d n=%d)", who, op->m, op->n);
    if (op->ens == CS_SRHT) {
        long long npad = 2;
        while (npad < op->n) npad *= 2;
        if (op->m > npad) return fail(c, CS_EINVAL, "%s: the Hadamard ensemble has at most %lld rows for n=%d (m=%d)", who, npad, op->n, op->m);
    }
    return CS_OK;
}

cs_status check_dict(cs_ctx* c, const cs_op* op, const cs_dict* dict, const char* who) {
    if (!dict) return fail(c, CS_EINVAL, "%s: dictionary is NULL", who);
    if (dict->G < 1 || dict->b < 1 || dict->rb < 1) return fail(c, CS_EINVAL, "%s: dictionary needs G, b, rb >= 1", who);
    if ((long long)dict->G * dict->b != op->n) return fail(c, CS_EINVAL, "%s: n (%d) != G*b (%d*%d)", who, op->n, dict->G, dict->b);
    if (!dict->psi && dict->rb != dict->b) return fail(c, CS_EINVAL, "%s: identity dictionary needs rb == b", who);
    if (dict->psi && dict->rb > dict->b) return fail(c, CS_EINVAL, "%s: rb > b", who);
    if (dict->psi && dict->rb > kMaxWeightedRb) return fail(c, CS_EINVAL, "%s: rb > %d with a dictionary is not supported", who, kMaxWeightedRb);
    if (dict->psi && !aligned16(dict->psi)) return fail(c, CS_EALIGN, "%s: psi is not 16-byte aligned", who);
    return CS_OK;
}

cs_status bind_device(cs_ctx* c) {
    hipError_t e = hipSetDevice(c->device);
    if (e != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    return CS_OK;
}

cs_status find_or_build_plan(cs_ctx* c, const cs_op* op, const cs_dict* dict, const Plan** out) {
    for (const PlanEntry& pe : c->plans) {
        if (pe.op.ens == op->ens && pe.op.seed == op->seed && pe.op.stream_id == op->stream_id &&
            pe.op.m == op->m && pe.op.n == op->n && pe.psi == dict->psi && pe.G == dict->G &&
            pe.b == dict->b && pe.rb == dict->rb) {
            *out = &pe.plan;
            return CS_OK;
        }
    }
    PlanEntry pe;
    pe.op = *op; pe.psi = dict->psi; pe.G = dict->G; pe.b = dict->b; pe.rb = dict->rb;
    Plan& p = pe.plan;
    p.op = make_desc(*op);
    p.G = dict->G; p.b = dict->b; p.rb = dict->rb;
    p.N = dict->G * dict->rb;
    p.weighted = dict->psi ? 1 : 0;
    p.Mt = nullptr; p.Mr = nullptr; p.gram = nullptr; p.W = nullptr;
    hipError_t e;
    if ((e = hipMalloc(&p.Mt, (size_t)p.N * op->m * sizeof(float))) != hipSuccess ||
        (e = hipMalloc(&p.Mr, (size_t)p.N * op->m * sizeof(float))) != hipSuccess ||
        (e = hipMalloc(&p.gram, (size_t)p.N * p.N * sizeof(float))) != hipSuccess ||
        (p.weighted && (e = hipMalloc(&p.W, (size_t)p.G * p.rb * p.rb * sizeof(float))) != hipSuccess)) {
        if (p.Mt) (void)hipFree(p.Mt);
        if (p.Mr) (void)hipFree(p.Mr);
        if (p.gram) (void)hipFree(p.gram);
        if (p.W) (void)hipFree(p.W);
        (void)hipGetLastError();
        return fail(c, CS_ENOMEM, "cs_plan: device allocation failed: %s", hipGetErrorString(e));
    }
    e = launch_plan_build(p, dict->psi, c->stream);
    if (e != hipSuccess) {
        (void)hipFree(p.Mt); (void)hipFree(p.Mr); (void)hipFree(p.gram);
        if (p.W) (void)hipFree(p.W);
        return hip_fail(c, e, "cs_plan: kernel launch");
    }
    c->plans.push_back(pe);
    *out = &c->plans.back().plan;
    return CS_OK;
}

cs_status check_recover_args(cs_ctx* c, const cs_op* op, const cs_dict* dict, int k, const char* who) {
    cs_status st;
    if ((st = check_op(c, op, who)) != CS_OK) return st;
    if ((st = check_dict(c, op, dict, who)) != CS_OK) return st;
    if (k < 1 || k > dict->G) return fail(c, CS_EINVAL, "%s: k=%d out of range [1, G=%d]", who, k, dict->G);
    if ((long long)k * dict->rb >= op->m)
        return fail(c, CS_EILLPOSED, "%s: k*rb = %lld >= m = %d, the refit is under-determined", who,
                    (long long)k * dict->rb, op->m);
    return CS_OK;
}

cs_status run_recover(cs_ctx* c, const cs_op* op, const cs_dict* dict, int k, const float* y, int B,
                      int32_t* support, float* coef, float* resid, float* margin, size_t scratch_off,
                      const char* who) {
    const Plan* plan = nullptr;
    cs_status st = find_or_build_plan(c, op, dict, &plan);
    if (st != CS_OK) return st;
    RecoverArgs a;
    a.y = y; a.B = B; a.k = k; a.support = support; a.coef = coef; a.resid = resid; a.margin = margin;
    a.spill_stride = recover_spill_floats(*plan, k, c->lds_limit);
    a.spill = nullptr;
    if (a.spill_stride) {
        const size_t need = scratch_off + a.spill_stride * sizeof(float) * (size_t)B;
        if (need > c->scratch_bytes)
            return fail(c, CS_ENOMEM, "%s: needs %zu bytes of scratch, context has %zu", who, need, c->scratch_bytes);
        a.spill = reinterpret_cast<float*>(static_cast<char*>(c->scratch) + scratch_off);
    }
    hipError_t e = launch_recover(*plan, a, c->lds_limit, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, who);
    return CS_OK;
}

}  // namespace

extern "C" {

cs_status cs_create(cs_ctx** out, int device, void* hip_stream, size_t scratch_bytes) {
    if (!out) return CS_EINVAL;
    *out = nullptr;
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || device < 0 || device >= ndev) { (void)hipGetLastError(); return CS_EHIP; }
    if ((e = hipSetDevice(device)) != hipSuccess) return CS_EHIP;
    if (device < kMaxDevices && !g_static_scratch[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return CS_EHIP; }
        g_static_scratch[device] = p;
    }
    cs_ctx* c = new (std::nothrow) cs_ctx();
    if (!c) return CS_ENOMEM;
    c->err[0] = 0;
    c->device = device;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->scratch_bytes = scratch_bytes ? scratch_bytes : kDefaultScratch;
    c->scratch = nullptr;
    if (hipMalloc(&c->scratch, c->scratch_bytes) != hipSuccess) {
        (void)hipGetLastError();
        delete c;
        return CS_ENOMEM;
    }
    int lds = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess || lds <= 0)
        lds = 64 * 1024;
    c->lds_limit = lds;
    *out = c;
    return CS_OK;
}

void cs_destroy(cs_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    for (PlanEntry& pe : c->plans) {
        if (pe.plan.Mt) (void)hipFree(pe.plan.Mt);
        if (pe.plan.Mr) (void)hipFree(pe.plan.Mr);
        if (pe.plan.gram) (void)hipFree(pe.plan.gram);
        if (pe.plan.W) (void)hipFree(pe.plan.W);
    }
    for (cs_ctx::PlanGroup& g : c->groups)
        if (g.d_plans) (void)hipFree(g.d_plans);
    if (c->scratch) (void)hipFree(c->scratch);
    delete c;
}

const char* cs_last_error(const cs_ctx* c) { return c ? c->err : "no context"; }

cs_status cs_set_stream(cs_ctx* c, void* hip_stream) {
    if (!c) return CS_EINVAL;
    c->stream = static_cast<hipStream_t>(hip_stream);
    return CS_OK;
}

cs_status cs_set_union_hint(cs_ctx* c, int hint) {
    if (!c) return CS_EINVAL;
    if (hint != CS_UNION_AUTO && hint != CS_UNION_DENSE && hint != CS_UNION_SPARSE)
        return fail(c, CS_EINVAL, "cs_set_union_hint: unknown hint %d", hint);
    c->union_hint = hint;
    return CS_OK;
}

cs_status cs_plan(cs_ctx* c, const cs_op* op, const cs_dict* dict) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    cs_status st;
    if ((st = check_op(c, op, "cs_plan")) != CS_OK) return st;
    if ((st = check_dict(c, op, dict, "cs_plan")) != CS_OK) return st;
    if ((st = bind_device(c)) != CS_OK) return st;
    const Plan* plan = nullptr;
    return find_or_build_plan(c, op, dict, &plan);
    });
}

cs_status cs_plan_drop(cs_ctx* c, const cs_op* op, const cs_dict* dict) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    if (!op || !dict) return fail(c, CS_EINVAL, "cs_plan_drop: NULL operator or dictionary");
    cs_status st;
    if ((st = bind_device(c)) != CS_OK) return st;
    for (size_t i = 0; i < c->plans.size(); ++i) {
        const PlanEntry& pe = c->plans[i];
        if (!(pe.op.ens == op->ens && pe.op.seed == op->seed && pe.op.stream_id == op->stream_id &&
              pe.op.m == op->m && pe.op.n == op->n && pe.psi == dict->psi && pe.G == dict->G &&
              pe.b == dict->b && pe.rb == dict->rb))
            continue;
        // work that reads the plan may still be queued
        hipError_t e = hipStreamSynchronize(c->stream);
        if (e != hipSuccess) return hip_fail(c, e, "cs_plan_drop: stream synchronisation");
        const float* atoms = pe.plan.Mt;
        for (size_t g = 0; g < c->groups.size();) {           // device tables that list this plan go with it
            bool uses = false;
            for (const float* key : c->groups[g].key) uses = uses || key == atoms;
            if (uses) {
                if (c->groups[g].d_plans) (void)hipFree(c->groups[g].d_plans);
                c->groups.erase(c->groups.begin() + (long)g);
            } else {
                ++g;
            }
        }
        if (pe.plan.Mt) (void)hipFree(pe.plan.Mt);
        if (pe.plan.Mr) (void)hipFree(pe.plan.Mr);
        if (pe.plan.gram) (void)hipFree(pe.plan.gram);
        if (pe.plan.W) (void)hipFree(pe.plan.W);
        c->plans.erase(c->plans.begin() + (long)i);
        return CS_OK;
    }
    return CS_OK;                                             // nothing cached: nothing to do
    });
}

cs_status cs_sketch(cs_ctx* c, const cs_op* op, const float* z, int B, float* y) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    cs_status st;
    if ((st = check_op(c, op, "cs_sketch")) != CS_OK) return st;
    if (B < 0) return fail(c, CS_EINVAL, "cs_sketch: B < 0");
    if (B == 0) return CS_OK;
    if (!z || !y) return fail(c, CS_EINVAL, "cs_sketch: NULL buffer");
    if (!aligned16(z) || !aligned16(y)) return fail(c, CS_EALIGN, "cs_sketch: buffer not 16-byte aligned");
    if ((st = bind_device(c)) != CS_OK) return st;
    if (op->ens == CS_SRHT && !sketch_srht_supported(make_desc(*op)))
        return fail(c, CS_EINVAL, "cs_sketch: the Hadamard ensemble is limited to n <= 32768 (n=%d)", op->n);
    hipError_t e = launch_sketch(make_desc(*op), z, B, y, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_sketch");
    return CS_OK;
    });
}

cs_status cs_sketch_multi(cs_ctx* c, int n_ops, const cs_op* ops, const float* z, int B, float* y) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    if (n_ops < 1 || n_ops > 65535) return fail(c, CS_EINVAL, "cs_sketch_multi: n_ops=%d out of range [1, 65535]", n_ops);
    if (!ops) return fail(c, CS_EINVAL, "cs_sketch_multi: NULL operator list");
    cs_status st;
    for (int j = 0; j < n_ops; ++j) {
        if ((st = check_op(c, &ops[j], "cs_sketch_multi")) != CS_OK) return st;
        if (ops[j].ens != ops[0].ens || ops[j].m != ops[0].m || ops[j].n != ops[0].n)
            return fail(c, CS_EINVAL, "cs_sketch_multi: operator %d differs in ensemble or shape from operator 0", j);
    }
    if (B < 0) return fail(c, CS_EINVAL, "cs_sketch_multi: B < 0");
    if (B == 0) return CS_OK;
    if (!z || !y) return fail(c, CS_EINVAL, "cs_sketch_multi: NULL buffer");
    if (!aligned16(z) || !aligned16(y)) return fail(c, CS_EALIGN, "cs_sketch_multi: buffer not 16-byte aligned");
    if ((st = bind_device(c)) != CS_OK) return st;
    std::vector<OpDesc> descs((size_t)n_ops);
    for (int j = 0; j < n_ops; ++j) descs[(size_t)j] = make_desc(ops[j]);
    if (ops[0].ens == CS_SRHT && !sketch_srht_supported(descs[0]))
        return fail(c, CS_EINVAL, "cs_sketch_multi: the Hadamard ensemble is limited to n <= 32768 (n=%d)", ops[0].n);
    hipError_t e = launch_sketch_multi(descs.data(), n_ops, z, B, y, c->stream, c->scratch, c->scratch_bytes);
    if (e != hipSuccess) return hip_fail(c, e, "cs_sketch_multi");
    return CS_OK;
    });
}

cs_status cs_recover_support(cs_ctx* c, const cs_op* op, const cs_dict* dict, int k,
                             const float* y, int B,
                             int32_t* support, float* coef, float* resid_norm, float* margin) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    cs_status st;
    if ((st = check_recover_args(c, op, dict, k, "cs_recover_support")) != CS_OK) return st;
    if (B < 0) return fail(c, CS_EINVAL, "cs_recover_support: B < 0");
    if (B == 0) return CS_OK;
    if (!y || !support) return fail(c, CS_EINVAL, "cs_recover_support: NULL buffer");
    if (!aligned16(y) || !aligned16(support) || !aligned16(coef) || !aligned16(resid_norm) || !aligned16(margin))
        return fail(c, CS_EALIGN, "cs_recover_support: buffer not 16-byte aligned");
    if ((st = bind_device(c)) != CS_OK) return st;
    return run_recover(c, op, dict, k, y, B, support, coef, resid_norm, margin, 0, "cs_recover_support");
    });
}

cs_status cs_recover_support_multi(cs_ctx* c, int n_ops, const cs_op* ops, const cs_dict* dicts, int k,
                                   const float* y, int B,
                                   int32_t* support, float* coef, float* resid_norm, float* margin) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    if (n_ops < 1 || n_ops > 65535) return fail(c, CS_EINVAL, "cs_recover_support_multi: n_ops=%d out of range [1, 65535]", n_ops);
    if (!ops || !dicts) return fail(c, CS_EINVAL, "cs_recover_support_multi: NULL operator or dictionary list");
    cs_status st;
    for (int j = 0; j < n_ops; ++j) {
        if ((st = check_recover_args(c, &ops[j], &dicts[j], k, "cs_recover_support_multi")) != CS_OK) return st;
        if (ops[j].m != ops[0].m || ops[j].n != ops[0].n || dicts[j].G != dicts[0].G || dicts[j].b != dicts[0].b ||
            dicts[j].rb != dicts[0].rb || (dicts[j].psi == nullptr) != (dicts[0].psi == nullptr))
            return fail(c, CS_EINVAL, "cs_recover_support_multi: operator %d differs in shape from operator 0", j);
    }
    if (B < 0) return fail(c, CS_EINVAL, "cs_recover_support_multi: B < 0");
    if (B == 0) return CS_OK;
    if (!y || !support) return fail(c, CS_EINVAL, "cs_recover_support_multi: NULL buffer");
    if (!aligned16(y) || !aligned16(support) || !aligned16(coef) || !aligned16(resid_norm) || !aligned16(margin))
        return fail(c, CS_EALIGN, "cs_recover_support_multi: buffer not 16-byte aligned");
    if ((st = bind_device(c)) != CS_OK) return st;
    std::vector<Plan> host_plans((size_t)n_ops);
    std::vector<const float*> key((size_t)n_ops);
    for (int j = 0; j < n_ops; ++j) {
        const Plan* pl = nullptr;
        if ((st = find_or_build_plan(c, &ops[j], &dicts[j], &pl)) != CS_OK) return st;
        host_plans[(size_t)j] = *pl;                    // the cache may move its entries; the device buffers stay
        key[(size_t)j] = pl->Mt;
    }
    const Plan* d_plans = nullptr;
    for (const cs_ctx::PlanGroup& g : c->groups)
        if (g.key == key) { d_plans = g.d_plans; break; }
    if (!d_plans) {                                     // first use of this list of operators: cold, like cs_plan
        Plan* dp = nullptr;
        hipError_t e = hipMalloc(&dp, sizeof(Plan) * (size_t)n_ops);
        if (e != hipSuccess) { (void)hipGetLastError(); return fail(c, CS_ENOMEM, "cs_recover_support_multi: device allocation failed"); }
        e = hipMemcpy(dp, host_plans.data(), sizeof(Plan) * (size_t)n_ops, hipMemcpyHostToDevice);
        if (e != hipSuccess) { (void)hipFree(dp); return hip_fail(c, e, "cs_recover_support_multi: upload of the plan list"); }
        c->groups.push_back({key, dp});
        d_plans = dp;
    }
    RecoverArgs a;
    a.y = y; a.B = B; a.k = k; a.support = support; a.coef = coef; a.resid = resid_norm; a.margin = margin;
    a.plans = d_plans; a.nplans = n_ops;
    a.spill_stride = recover_spill_floats(host_plans[0], k, c->lds_limit);
    a.spill = nullptr;
    if (a.spill_stride) {
        const size_t need = a.spill_stride * sizeof(float) * (size_t)B * (size_t)n_ops;
        if (need > c->scratch_bytes)
            return fail(c, CS_ENOMEM, "cs_recover_support_multi: needs %zu bytes of scratch, context has %zu", need, c->scratch_bytes);
        a.spill = reinterpret_cast<float*>(c->scratch);
    }
    hipError_t e = launch_recover(host_plans[0], a, c->lds_limit, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_recover_support_multi");
    return CS_OK;
    });
}

cs_status cs_recover_support_iht(cs_ctx* c, const cs_op* op, const cs_dict* dict, int k, int iters,
                                 const float* y, int B,
                                 int32_t* support, float* coef, float* resid_norm, float* margin) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    cs_status st;
    if ((st = check_recover_args(c, op, dict, k, "cs_recover_support_iht")) != CS_OK) return st;
    if (iters < 1) return fail(c, CS_EINVAL, "cs_recover_support_iht: iters < 1");
    if (B < 0) return fail(c, CS_EINVAL, "cs_recover_support_iht: B < 0");
    if (B == 0) return CS_OK;
    if (!y || !support) return fail(c, CS_EINVAL, "cs_recover_support_iht: NULL buffer");
    if (!aligned16(y) || !aligned16(support) || !aligned16(coef) || !aligned16(resid_norm) || !aligned16(margin))
        return fail(c, CS_EALIGN, "cs_recover_support_iht: buffer not 16-byte aligned");
    if ((st = bind_device(c)) != CS_OK) return st;
    const Plan* plan = nullptr;
    if ((st = find_or_build_plan(c, op, dict, &plan)) != CS_OK) return st;
    if (!recover_iht_supported(*plan, k, c->lds_limit))
        return fail(c, CS_EINVAL, "cs_recover_support_iht: needs rb == 1, k <= 64 and G <= 512");
    RecoverArgs a;
    a.y = y; a.B = B; a.k = k; a.support = support; a.coef = coef; a.resid = resid_norm; a.margin = margin;
    a.spill = nullptr; a.spill_stride = 0;
    hipError_t e = launch_recover_iht(*plan, a, iters, c->lds_limit, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_recover_support_iht");
    return CS_OK;
    });
}

cs_status cs_recover_support_inc(cs_ctx* c, const cs_op* op, const cs_dict* dict, int k,
                                 const float* y, int B,
                                 const int32_t* prev_support, const float* prev_coef, float gamma, int swaps,
                                 int32_t* support, float* coef, float* resid_norm, float* margin) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    cs_status st;
    if ((st = check_recover_args(c, op, dict, k, "cs_recover_support_inc")) != CS_OK) return st;
    if (swaps < 0 || swaps > k) return fail(c, CS_EINVAL, "cs_recover_support_inc: swaps=%d out of range [0, k=%d]", swaps, k);
    if (!(gamma >= 0.f)) return fail(c, CS_EINVAL, "cs_recover_support_inc: gamma must be >= 0");
    if (B < 0) return fail(c, CS_EINVAL, "cs_recover_support_inc: B < 0");
    if (B == 0) return CS_OK;
    if (!y || !support || !prev_support) return fail(c, CS_EINVAL, "cs_recover_support_inc: NULL buffer");
    if (!aligned16(y) || !aligned16(support) || !aligned16(coef) || !aligned16(resid_norm) || !aligned16(margin) ||
        !aligned16(prev_support) || !aligned16(prev_coef))
        return fail(c, CS_EALIGN, "cs_recover_support_inc: buffer not 16-byte aligned");
    if ((st = bind_device(c)) != CS_OK) return st;
    const Plan* plan = nullptr;
    if ((st = find_or_build_plan(c, op, dict, &plan)) != CS_OK) return st;
    if (!recover_inc_supported(*plan, k, c->lds_limit))
        return fail(c, CS_EINVAL, "cs_recover_support_inc: needs rb == 1, k <= 64 and G <= 512");
    RecoverArgs a;
    a.y = y; a.B = B; a.k = k; a.support = support; a.coef = coef; a.resid = resid_norm; a.margin = margin;
    a.spill = nullptr; a.spill_stride = 0;
    IncArgs q;
    q.prev_support = prev_support; q.prev_coef = prev_coef; q.gamma = gamma; q.swaps = swaps;
    hipError_t e = launch_recover_inc(*plan, a, q, c->lds_limit, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_recover_support_inc");
    return CS_OK;
    });
}

size_t cs_inc_state_words(int k) { return k < 1 ? 0 : recover_inc_state_words(k); }

cs_status cs_recover_support_inc_carry(cs_ctx* c, const cs_op* op, const cs_dict* dict, int k,
                                       const float* y, int B,
                                       const int32_t* prev_support, int swaps, uint32_t* state,
                                       int32_t* support, float* coef, float* resid_norm, float* margin) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    cs_status st;
    if ((st = check_recover_args(c, op, dict, k, "cs_recover_support_inc_carry")) != CS_OK) return st;
    if (swaps < 0 || swaps > k) return fail(c, CS_EINVAL, "cs_recover_support_inc_carry: swaps=%d out of range [0, k=%d]", swaps, k);
    if (B < 0) return fail(c, CS_EINVAL, "cs_recover_support_inc_carry: B < 0");
    if (B == 0) return CS_OK;
    if (!y || !support || !prev_support || !state) return fail(c, CS_EINVAL, "cs_recover_support_inc_carry: NULL buffer");
    if (!aligned16(y) || !aligned16(support) || !aligned16(coef) || !aligned16(resid_norm) || !aligned16(margin) ||
        !aligned16(prev_support) || !aligned16(state))
        return fail(c, CS_EALIGN, "cs_recover_support_inc_carry: buffer not 16-byte aligned");
    if ((st = bind_device(c)) != CS_OK) return st;
    const Plan* plan = nullptr;
    if ((st = find_or_build_plan(c, op, dict, &plan)) != CS_OK) return st;
    if (!recover_inc_supported(*plan, k, c->lds_limit))
        return fail(c, CS_EINVAL, "cs_recover_support_inc_carry: needs rb == 1, k <= 64 and G <= 512");
    RecoverArgs a;
    a.y = y; a.B = B; a.k = k; a.support = support; a.coef = coef; a.resid = resid_norm; a.margin = margin;
    a.spill = nullptr; a.spill_stride = 0;
    IncArgs q;
    q.prev_support = prev_support; q.prev_coef = nullptr; q.gamma = 0.f; q.swaps = swaps;
    q.state = state; q.state_stride = recover_inc_state_words(k);
    hipError_t e = launch_recover_carry(*plan, a, q, c->lds_limit, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_recover_support_inc_carry");
    return CS_OK;
    });
}

static cs_status block_ffn_with_scratch(cs_ctx* c, int dtype, const void* Wg, const void* Wu, const void* Wd,
                                        int d, int G, int b, const void* x, int T,
                                        const int32_t* support, int k, int shared, void* out,
                                        void* work, size_t work_bytes, const char* work_name) {
    return guarded(c, [&]() -> cs_status {
    if (dtype != CS_F32 && dtype != CS_BF16) return fail(c, CS_EINVAL, "cs_block_ffn: unknown dtype %d", dtype);
    if (d < 8 || (d % 8) || b < 8 || (b % 8) || G < 1) return fail(c, CS_EINVAL, "cs_block_ffn: need d %% 8 == 0, b %% 8 == 0, G >= 1");
    if (k < 0 || k > G) return fail(c, CS_EINVAL, "cs_block_ffn: k=%d out of range [0, G=%d]", k, G);
    if (T < 0 || T > 65535) return fail(c, CS_EINVAL, "cs_block_ffn: T=%d out of range [0, 65535]", T);
    if (T == 0) return CS_OK;
    if (!Wg || !Wu || !Wd || !x || !out || (k > 0 && !support)) return fail(c, CS_EINVAL, "cs_block_ffn: NULL buffer");
    if (!aligned16(Wg) || !aligned16(Wu) || !aligned16(Wd) || !aligned16(x) || !aligned16(out) || !aligned16(support))
        return fail(c, CS_EALIGN, "cs_block_ffn: buffer not 16-byte aligned");
    cs_status st;
    if ((st = bind_device(c)) != CS_OK) return st;
    const size_t esz = dtype == CS_F32 ? 4 : 2;
    if (k == 0) {
        hipError_t e = launch_zero_fill(out, (size_t)T * d * esz, c->stream);
        if (e != hipSuccess) return hip_fail(c, e, "cs_block_ffn");
        return CS_OK;
    }
    FfnArgs a;
    a.dtype = dtype; a.Wg = Wg; a.Wu = Wu; a.Wd = Wd; a.d = d; a.G = G; a.b = b;
    a.x = x; a.T = T; a.support = support; a.k = k; a.shared = shared ? 1 : 0; a.out = out;
    a.scratch = work; a.scratch_bytes = work_bytes;
    a.union_hint = c->union_hint;
    const size_t need = ffn_scratch_bytes(a);
    if (need > work_bytes)
        return fail(c, CS_ENOMEM, "cs_block_ffn: needs %zu bytes of scratch, %s has %zu", need, work_name, work_bytes);
    hipError_t e = launch_block_ffn(a, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_block_ffn");
    return CS_OK;
    });
}

cs_status cs_block_ffn(cs_ctx* c, int dtype, const void* Wg, const void* Wu, const void* Wd,
                       int d, int G, int b, const void* x, int T,
                       const int32_t* support, int k, int shared, void* out) {
    if (!c) return CS_EINVAL;
    return block_ffn_with_scratch(c, dtype, Wg, Wu, Wd, d, G, b, x, T, support, k, shared, out,
                                  c->scratch, c->scratch_bytes, "the context");
}

cs_status cs_block_ffn_static(cs_ctx* c, int dtype, const void* Wg, const void* Wu, const void* Wd,
                              int d, int G, int b, const void* x, int T,
                              const int32_t* support, int k, int shared, void* out) {
    if (!c) return CS_EINVAL;
    void* work = c->device < kMaxDevices ? g_static_scratch[c->device] : nullptr;
    if (!work) return fail(c, CS_EHIP, "cs_block_ffn_static: no static workspace on device %d", c->device);
    return block_ffn_with_scratch(c, dtype, Wg, Wu, Wd, d, G, b, x, T, support, k, shared, out,
                                  work, (size_t)CS_STATIC_SCRATCH_BYTES, "the static workspace");
}

cs_status cs_head_attn(cs_ctx* c, int dtype, const void* q, const void* K, const void* V,
                       int B, int H, int L, int dh, const int32_t* heads, int kh, void* out) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    if (dtype != CS_F32 && dtype != CS_BF16) return fail(c, CS_EINVAL, "cs_head_attn: unknown dtype %d", dtype);
    if (dh != 64 && dh != 128 && dh != 256) return fail(c, CS_EINVAL, "cs_head_attn: dh must be 64, 128 or 256");
    if (H < 1 || L < 1) return fail(c, CS_EINVAL, "cs_head_attn: need H >= 1 and L >= 1");
    if (kh < 0 || kh > H) return fail(c, CS_EINVAL, "cs_head_attn: kh=%d out of range [0, H=%d]", kh, H);
    if (B < 0 || B > 65535 || H > 65535) return fail(c, CS_EINVAL, "cs_head_attn: B or H out of range");
    if (B == 0) return CS_OK;
    if (!q || !K || !V || !out || (kh > 0 && !heads)) return fail(c, CS_EINVAL, "cs_head_attn: NULL buffer");
    if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(out) || !aligned16(heads))
        return fail(c, CS_EALIGN, "cs_head_attn: buffer not 16-byte aligned");
    cs_status st;
    if ((st = bind_device(c)) != CS_OK) return st;
    AttnArgs a;
    a.dtype = dtype; a.q = q; a.K = K; a.V = V; a.B = B; a.H = H; a.L = L; a.dh = dh;
    a.heads = heads; a.kh = kh; a.out = out; a.scratch = c->scratch; a.scratch_bytes = c->scratch_bytes;
    const size_t need = attn_scratch_bytes(a);
    if (need > c->scratch_bytes)
        return fail(c, CS_ENOMEM, "cs_head_attn: needs %zu bytes of scratch, context has %zu", need, c->scratch_bytes);
    hipError_t e = launch_head_attn(a, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_head_attn");
    return CS_OK;
    });
}

cs_status cs_joint_select(cs_ctx* c, const cs_op* tok_op, const float* y_tok, int k_tok,
                          const cs_op* ch_op, const cs_dict* ch_dict, const float* y_ch, int k_ch,
                          int32_t* tokens, int32_t* support, float* resid_norm, float* margin) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    cs_status st;
    if ((st = check_op(c, tok_op, "cs_joint_select(tokens)")) != CS_OK) return st;
    if (k_tok < 1 || k_tok > tok_op->n) return fail(c, CS_EINVAL, "cs_joint_select: k_tok=%d out of range [1, n=%d]", k_tok, tok_op->n);
    if ((st = check_recover_args(c, ch_op, ch_dict, k_ch, "cs_joint_select(channels)")) != CS_OK) return st;
    if (!y_tok || !y_ch || !tokens || !support) return fail(c, CS_EINVAL, "cs_joint_select: NULL buffer");
    if (!aligned16(y_tok) || !aligned16(y_ch) || !aligned16(tokens) || !aligned16(support) ||
        !aligned16(resid_norm) || !aligned16(margin))
        return fail(c, CS_EALIGN, "cs_joint_select: buffer not 16-byte aligned");
    if ((st = bind_device(c)) != CS_OK) return st;
    const size_t proxy_bytes = (((size_t)tok_op->n * sizeof(float)) + 255) & ~(size_t)255;
    if (proxy_bytes > c->scratch_bytes)
        return fail(c, CS_ENOMEM, "cs_joint_select: needs %zu bytes of scratch, context has %zu", proxy_bytes, c->scratch_bytes);
    float* proxy = reinterpret_cast<float*>(c->scratch);
    hipError_t e = launch_backproject(make_desc(*tok_op), y_tok, proxy, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_joint_select: back-projection");
    e = launch_topk(proxy, tok_op->n, k_tok, tokens, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_joint_select: top-k");
    return run_recover(c, ch_op, ch_dict, k_ch, y_ch, 1, support, nullptr, resid_norm, margin, proxy_bytes,
                       "cs_joint_select: recovery");
    });
}

cs_status cs_joint_select_coupled(cs_ctx* c, const cs_op* tok_op, const float* y_tok, int k_tok,
                                  const cs_op* ch_op, const cs_dict* ch_dict, const float* Y_ch, int k_ch,
                                  int32_t* tokens, int32_t* support, float* ybar,
                                  float* resid_norm, float* margin) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    cs_status st;
    if ((st = check_op(c, tok_op, "cs_joint_select_coupled(tokens)")) != CS_OK) return st;
    if (k_tok < 1 || k_tok > tok_op->n)
        return fail(c, CS_EINVAL, "cs_joint_select_coupled: k_tok=%d out of range [1, n=%d]", k_tok, tok_op->n);
    if ((st = check_recover_args(c, ch_op, ch_dict, k_ch, "cs_joint_select_coupled(channels)")) != CS_OK) return st;
    if (!y_tok || !Y_ch || !tokens || !support) return fail(c, CS_EINVAL, "cs_joint_select_coupled: NULL buffer");
    if (!aligned16(y_tok) || !aligned16(Y_ch) || !aligned16(tokens) || !aligned16(support) || !aligned16(ybar) ||
        !aligned16(resid_norm) || !aligned16(margin))
        return fail(c, CS_EALIGN, "cs_joint_select_coupled: buffer not 16-byte aligned");
    if ((st = bind_device(c)) != CS_OK) return st;
    // scratch: token proxy | chunk sums of the pooled sketch | pooled sketch | recovery workspace
    const size_t proxy_bytes = (((size_t)tok_op->n * sizeof(float)) + 255) & ~(size_t)255;
    const size_t part_bytes = ((pool_rows_scratch_floats(ch_op->m, k_tok) * sizeof(float)) + 255) & ~(size_t)255;
    const size_t ybar_bytes = (((size_t)ch_op->m * sizeof(float)) + 255) & ~(size_t)255;
    const size_t used = proxy_bytes + part_bytes + ybar_bytes;
    if (used > c->scratch_bytes)
        return fail(c, CS_ENOMEM, "cs_joint_select_coupled: needs %zu bytes of scratch, context has %zu", used, c->scratch_bytes);
    char* base = static_cast<char*>(c->scratch);
    float* proxy = reinterpret_cast<float*>(base);
    float* partial = reinterpret_cast<float*>(base + proxy_bytes);
    float* pooled = reinterpret_cast<float*>(base + proxy_bytes + part_bytes);
    hipError_t e = launch_backproject(make_desc(*tok_op), y_tok, proxy, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_joint_select_coupled: back-projection");
    e = launch_topk(proxy, tok_op->n, k_tok, tokens, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_joint_select_coupled: top-k");
    e = launch_pool_rows(Y_ch, tok_op->n, ch_op->m, tokens, k_tok, partial, pooled, ybar, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_joint_select_coupled: pooling");
    return run_recover(c, ch_op, ch_dict, k_ch, pooled, 1, support, nullptr, resid_norm, margin, used,
                       "cs_joint_select_coupled: recovery");
    });
}

cs_status cs_softmax_entropy(cs_ctx* c, const float* logits, int B, int V, float* entropy) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    if (B < 0 || B > 65535) return fail(c, CS_EINVAL, "cs_softmax_entropy: B out of range [0, 65535]");
    if (V < 1) return fail(c, CS_EINVAL, "cs_softmax_entropy: V < 1");
    if (B == 0) return CS_OK;
    if (!logits || !entropy) return fail(c, CS_EINVAL, "cs_softmax_entropy: NULL buffer");
    if (!aligned16(logits) || !aligned16(entropy)) return fail(c, CS_EALIGN, "cs_softmax_entropy: buffer not 16-byte aligned");
    cs_status st;
    if ((st = bind_device(c)) != CS_OK) return st;
    const size_t need = softmax_entropy_scratch_floats(B, V) * sizeof(float);
    if (need > c->scratch_bytes)
        return fail(c, CS_ENOMEM, "cs_softmax_entropy: needs %zu bytes of scratch, context has %zu", need, c->scratch_bytes);
    hipError_t e = launch_softmax_entropy(logits, B, V, reinterpret_cast<float*>(c->scratch), entropy, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_softmax_entropy");
    return CS_OK;
    });
}

cs_status cs_stream_read(cs_ctx* c, const void* src, size_t bytes, uint32_t* checksum) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    if (bytes == 0) return CS_OK;
    if (!src || !checksum) return fail(c, CS_EINVAL, "cs_stream_read: NULL buffer");
    if (!aligned16(src) || (reinterpret_cast<uintptr_t>(checksum) & 3u))
        return fail(c, CS_EALIGN, "cs_stream_read: src must be 16-byte aligned, checksum 4-byte aligned");
    cs_status st;
    if ((st = bind_device(c)) != CS_OK) return st;
    hipError_t e = launch_stream_read(src, bytes, checksum, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_stream_read");
    return CS_OK;
    });
}

int32_t cs_uds_budget(int32_t m_base, float gamma, float entropy, int32_t m_min, int32_t m_max) {
    if (m_min > m_max || m_min < 1 || !std::isfinite(gamma) || !std::isfinite(entropy)) return -1;
    const double v = std::floor((double)m_base * (1.0 + (double)gamma * (double)entropy));
    if (v < (double)m_min) return m_min;
    if (v > (double)m_max) return m_max;
    return (int32_t)v;
}

cs_status cs_gather_rows(cs_ctx* c, int dtype, const void* x, int n_rows, int d,
                         const int32_t* tokens, int k_tok, void* out) {
    if (!c) return CS_EINVAL;
    return guarded(c, [&]() -> cs_status {
    if (dtype != CS_F32 && dtype != CS_BF16) return fail(c, CS_EINVAL, "cs_gather_rows: unknown dtype %d", dtype);
    if (d < 8 || (d % 8) || n_rows < 1) return fail(c, CS_EINVAL, "cs_gather_rows: need d %% 8 == 0 and n_rows >= 1");
    if (k_tok < 0 || k_tok > 65535 * 1024) return fail(c, CS_EINVAL, "cs_gather_rows: k_tok out of range");
    if (k_tok == 0) return CS_OK;
    if (!x || !tokens || !out) return fail(c, CS_EINVAL, "cs_gather_rows: NULL buffer");
    if (!aligned16(x) || !aligned16(tokens) || !aligned16(out)) return fail(c, CS_EALIGN, "cs_gather_rows: buffer not 16-byte aligned");
    cs_status st;
    if ((st = bind_device(c)) != CS_OK) return st;
    hipError_t e = launch_gather_rows(x, n_rows, (size_t)d * (dtype == CS_F32 ? 4 : 2), tokens, k_tok, out, c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "cs_gather_rows");
    return CS_OK;
    });
}

}  // extern "C"
