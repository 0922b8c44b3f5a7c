// Sanitizer driver of the library's HOST code (test infrastructure, CPU only).  tests/test_sanitizers.py compiles
// every file under csrc/ for the host alone under -fsanitize=address,undefined and links the objects with this file,
// which stands in for the HIP runtime: the few entry points the library names (kernel launch, occupancy query, events,
// the status-word copy) are inert counters, so no GPU and no runtime is involved and no kernel runs.  What runs for
// real is all host code of the library: argument validation, the workspace layouts, pointer arithmetic on the
// workspace, the choice of kernels, split factors and grid sizes, and the profiling bookkeeping, over a sweep of valid
// and invalid descriptors, with the sanitizers watching.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <vector>

#include "cce_kernels.hpp"  // ProfScope
#include "cce_neg.h"

static int g_launches = 0;

// HIP runtime entry points named by the library: inert stand-ins
extern "C" {
void **__hipRegisterFatBinary(const void *) { static void *h; return &h; }
void __hipRegisterFunction(void **, const void *, char *, const char *, unsigned, void *, void *, void *, void *, int *) {}
void __hipUnregisterFatBinary(void **) {}
hipError_t __hipPushCallConfiguration(dim3, dim3, size_t, hipStream_t) { return hipSuccess; }
hipError_t __hipPopCallConfiguration(dim3 *, dim3 *, size_t *, hipStream_t *) { return hipSuccess; }
hipError_t hipLaunchKernel(const void *, dim3, dim3, void **, size_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
void __hipRegisterVar(void **, void *, char *, char *, int, size_t, int, int) {}
hipError_t hipGetSymbolAddress(void **p, const void *) { alignas(256) static char stand_in[256]; *p = stand_in; return hipSuccess; }
hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
hipError_t hipDeviceGetAttribute(int *v, hipDeviceAttribute_t, int) { *v = 256; return hipSuccess; }
hipError_t hipOccupancyMaxActiveBlocksPerMultiprocessor(int *n, const void *, int, size_t) { *n = 2; return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t *e) { static char slots[4096]; static int n; *e = (hipEvent_t)&slots[n++ % 4096]; return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.25f; return hipSuccess; }
hipError_t hipMemcpyAsync(void *dst, const void *, size_t n, hipMemcpyKind, hipStream_t) { std::memset(dst, 0, n); return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
}

#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); return 1; } } while (0)

static cce_desc desc_of(int64_t N, int64_t V, int d, int K, int in_dt, int mode)
{
    cce_desc x;
    std::memset(&x, 0, sizeof x);
    x.N = N; x.V = V; x.d = d; x.K = K; x.in_dtype = in_dt; x.dH_dtype = CCE_F32; x.neg_mode = mode;
    x.mask_target_collisions = 1;
    return x;
}

int main()
{
    // "device" pointers are never dereferenced by host code: any aligned address will do
    alignas(256) static char arena[1 << 16];
    void *fake = arena;
    const int32_t *ids = reinterpret_cast<const int32_t *>(arena);
    float *fl = reinterpret_cast<float *>(arena);
    int calls = 0;
    const int64_t Ns[] = {0, 1, 77, 512, 51200, 204800};
    const int64_t Vs[] = {1, 157, 50000, 5000000};
    const int ds[] = {8, 64, 72, 128, 256, 320, 512};
    const int Ks[] = {0, 1, 130, 1024, 4096};
    for (int64_t N : Ns) for (int64_t V : Vs) for (int d : ds) for (int K : Ks)
        for (int dt = 0; dt < 2; ++dt) for (int mode = 0; mode < 3; ++mode) for (int reuse = 0; reuse < 2; ++reuse) {
            cce_desc x = desc_of(N, V, d, K, dt, mode);
            x.reuse_forward_prep = reuse;
            x.dH_dtype = (dt == CCE_BF16 && ((N + K) & 1)) ? CCE_BF16 : CCE_F32;
            x.validate_indices = (int)((N + V) & 1);
            const size_t bytes = cce_neg_workspace_bytes(&x);
            CHECK(bytes >= 256);
            CHECK(cce_neg_forward(&x, fake, fake, ids, ids, nullptr, fl, fl, fake, bytes, nullptr) == CCE_OK);
            CHECK(cce_neg_backward(&x, fake, fake, ids, ids, (const uint8_t *)fake, fl, (N & 1) ? fl : nullptr, fake, fl, fake, bytes, nullptr) == CCE_OK);
            CHECK(cce_neg_forward(&x, fake, fake, ids, ids, nullptr, fl, fl, fake, bytes - 1, nullptr) == CCE_ERR_WORKSPACE);
            if (mode != CCE_NEG_FULL) {
                cce_sampler s;
                std::memset(&s, 0, sizeof s);
                s.kind = CCE_SAMPLER_UNIFORM; s.seed = 7; s.stream = 3;
                CHECK(cce_neg_forward_sampled(&x, &s, fake, fake, ids, nullptr, fl, fl, fake, bytes, nullptr) == CCE_OK);
                CHECK(cce_neg_backward_sampled(&x, &s, fake, fake, ids, nullptr, fl, fl, fake, fl, fake, bytes, nullptr) == CCE_OK);
                s.kind = CCE_SAMPLER_ALIAS;
                CHECK(cce_neg_forward_sampled(&x, &s, fake, fake, ids, nullptr, fl, fl, fake, bytes, nullptr) == CCE_ERR_NULL);
            }
            ++calls;
        }
    // invalid descriptors are refused by every entry point, and the size query answers 0
    struct Bad { int64_t N, V; int d, K, dt, mode; cce_status want; };
    const Bad bad[] = {{-1, 10, 64, 4, 0, 0, CCE_ERR_SHAPE}, {4, 0, 64, 4, 0, 0, CCE_ERR_SHAPE}, {4, 10, 12, 4, 0, 0, CCE_ERR_SHAPE},
                       {4, 10, 520, 4, 0, 0, CCE_ERR_SHAPE}, {4, 10, 64, -2, 0, 0, CCE_ERR_SHAPE}, {4, 10, 64, 4, 9, 0, CCE_ERR_DTYPE},
                       {4, 10, 64, 4, 0, 5, CCE_ERR_SHAPE}, {4, (int64_t)1 << 31, 64, 4, 0, 0, CCE_ERR_SHAPE}};
    for (const Bad &b : bad) {
        cce_desc x = desc_of(b.N, b.V, b.d, b.K, b.dt, b.mode);
        CHECK(cce_neg_workspace_bytes(&x) == 0);
        CHECK(cce_neg_forward(&x, fake, fake, ids, ids, nullptr, fl, fl, fake, sizeof arena, nullptr) == b.want);
        CHECK(cce_neg_backward(&x, fake, fake, ids, ids, nullptr, fl, nullptr, fake, fl, fake, sizeof arena, nullptr) == b.want);
    }
    CHECK(cce_neg_workspace_bytes(nullptr) == 0);
    {   // the entry point on the library's own scratch: size limit, refusals, and a call that goes through
        cce_desc x = desc_of(2000000, 1000, 64, 256, CCE_BF16, CCE_NEG_SHARED);
        CHECK(cce_neg_forward_noalloc(&x, fake, fake, ids, ids, nullptr, fl, fl, nullptr) == CCE_ERR_WORKSPACE);
        x = desc_of(1000, 1000, 64, 256, CCE_BF16, CCE_NEG_SHARED);
        CHECK(cce_neg_forward_noalloc(&x, fake, fake, ids, ids, nullptr, fl, fl, nullptr) == CCE_OK);
        CHECK(cce_neg_forward_noalloc(&x, fake, fake, ids, nullptr, nullptr, fl, fl, nullptr) == CCE_ERR_NULL);
        x.validate_indices = 1;
        CHECK(cce_neg_forward_noalloc(&x, fake, fake, ids, ids, nullptr, fl, fl, nullptr) == CCE_ERR_UNSUPPORTED);
    }
    CHECK(cce_neg_forward(nullptr, fake, fake, ids, ids, nullptr, fl, fl, fake, 4096, nullptr) == CCE_ERR_NULL);
    cce_desc f = desc_of(256, 1000, 64, 0, CCE_BF16, CCE_NEG_FULL);
    f.filter_eps = 1e-4f;
    CHECK(cce_neg_workspace_bytes(&f) > 0);
    f.filter_eps = -1.f;
    CHECK(cce_neg_workspace_bytes(&f) == 0);
    // workspace helpers and the profiling bookkeeping
    CHECK(cce_neg_workspace_init(fake, 4096, nullptr) == CCE_OK);
    CHECK(cce_neg_workspace_init(arena + 4, 4096, nullptr) == CCE_ERR_WORKSPACE);
    CHECK(cce_neg_index_status(fake, 4096, nullptr) == CCE_OK);
    CHECK(cce_neg_index_status(fake, 8, nullptr) == CCE_ERR_WORKSPACE);
    CHECK(cce_neg_profile_enable(1) == CCE_OK);
    {
        cce::ProfScope a(cce::PROF_TILE_FWD, nullptr), b(cce::PROF_ITEM_DE, nullptr);
    }
    char names[3 * 32];
    float ms[3];
    int32_t n[3];
    CHECK(cce_neg_profile_read(1, names, ms, n) == 1);      // fewer slots than families: no write past the end
    { cce::ProfScope a(cce::PROF_TILE_FWD, nullptr), b(cce::PROF_ITEM_DE, nullptr), c(cce::PROF_PREP, nullptr); }
    CHECK(cce_neg_profile_read(3, names, ms, n) == 3 && n[0] == 1);
    CHECK(cce_neg_profile_enable(0) == CCE_OK);
    for (int s = CCE_OK; s <= CCE_ERR_HIP; ++s) CHECK(cce_status_string((cce_status)s) != nullptr);
    std::printf("ok %d descriptors, %d stub launches\n", calls, g_launches);
    return 0;
}
