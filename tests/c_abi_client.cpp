// A client of the C ABI that uses nothing but the HIP runtime and include/granq.h:
// no Python, no torch.  It runs the four calls on two of the hand-derived worked
// examples (tests/golden/worked_examples.txt: "batch_level_ranges", "signed_range")
// on a non-default stream and compares every output with the fixture values.
// Build: hipcc -I include tests/c_abi_client.cpp -L paper_2503_18339_amd -lgranq -o tests/c_abi_client
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "granq.h"

#define HIP_OK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    std::printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 2; } } while (0)
#define GRANQ_CHECK(call) do { granq_status_t s_ = (call); if (s_ != GRANQ_OK) { \
    std::printf("%s -> %s\n", #call, granq_status_string(s_)); return 3; } } while (0)

struct Case {
    const char *name;
    int bits;
    granq_desc_t desc;
    std::vector<float> x, mn, mx, s, z, xhat, mask;
    std::vector<unsigned char> codes;
};

template <typename T>
static int expect(const char *what, const char *name, const std::vector<T> &got, const std::vector<T> &want) {
    for (size_t i = 0; i < want.size(); ++i)
        if (!(got[i] == want[i])) {
            std::printf("%s: %s[%zu] = %g, expected %g\n", name, what, i, (double)got[i], (double)want[i]);
            return 1;
        }
    return 0;
}

static int run(const Case &cs, hipStream_t stream) {
    const size_t e = cs.x.size(), c = (size_t)cs.desc.c;
    float *x, *dy, *xhat, *dx, *mn, *mx, *s, *z;
    unsigned char *codes;
    void *ws;
    size_t ws_bytes = 0;
    GRANQ_CHECK(granq_workspace_bytes(&cs.desc, &ws_bytes));
    HIP_OK(hipMalloc(&x, e * 4)); HIP_OK(hipMalloc(&dy, e * 4)); HIP_OK(hipMalloc(&xhat, e * 4));
    HIP_OK(hipMalloc(&dx, e * 4)); HIP_OK(hipMalloc(&codes, e)); HIP_OK(hipMalloc(&ws, ws_bytes));
    HIP_OK(hipMalloc(&mn, c * 4)); HIP_OK(hipMalloc(&mx, c * 4)); HIP_OK(hipMalloc(&s, c * 4)); HIP_OK(hipMalloc(&z, c * 4));
    std::vector<float> hdy(e);
    for (size_t i = 0; i < e; ++i) hdy[i] = 1.0f + (float)i / 8.0f;
    HIP_OK(hipMemcpy(x, cs.x.data(), e * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dy, hdy.data(), e * 4, hipMemcpyHostToDevice));

    GRANQ_CHECK(granq_range_reduce(x, &cs.desc, mn, mx, ws, ws_bytes, stream));
    GRANQ_CHECK(granq_prescale(mn, mx, cs.desc.c, cs.bits, s, z, stream));
    GRANQ_CHECK(granq_fakequant_fwd(x, &cs.desc, s, z, cs.bits, xhat, codes, stream));
    GRANQ_CHECK(granq_fakequant_bwd(x, dy, &cs.desc, s, z, cs.bits, dx, stream));
    HIP_OK(hipStreamSynchronize(stream));

    std::vector<float> gmn(c), gmx(c), gs(c), gz(c), gxhat(e), gdx(e), wdx(e);
    std::vector<unsigned char> gcodes(e);
    HIP_OK(hipMemcpy(gmn.data(), mn, c * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gmx.data(), mx, c * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gs.data(), s, c * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gz.data(), z, c * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gxhat.data(), xhat, e * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gdx.data(), dx, e * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gcodes.data(), codes, e, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < e; ++i) wdx[i] = hdy[i] * cs.mask[i];
    int bad = expect("min", cs.name, gmn, cs.mn) + expect("max", cs.name, gmx, cs.mx) +
              expect("scale", cs.name, gs, cs.s) + expect("zero_point", cs.name, gz, cs.z) +
              expect("codes", cs.name, gcodes, cs.codes) + expect("x_hat", cs.name, gxhat, cs.xhat) +
              expect("dx", cs.name, gdx, wdx);
    void *all[] = {x, dy, xhat, dx, codes, ws, mn, mx, s, z};
    for (void *p : all) HIP_OK(hipFree(p));
    return bad;
}

int main() {
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0) { std::printf("no GPU\n"); return 4; }
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    // error paths need no GPU work
    granq_desc_t bad = {0, 1, 1, 1, GRANQ_F32};
    size_t n = 0;
    if (granq_workspace_bytes(&bad, &n) != GRANQ_ERR_INVALID_ARG) { std::printf("bad descriptor accepted\n"); return 5; }
    Case a = {"batch_level_ranges", 2, {2, 2, 1, 2, GRANQ_F32},
              {0, 3, -3, 0, 6, 1.5f, 1, 3}, {0, -3}, {6, 3}, {2, 2}, {0, 2},
              {0, 4, -4, 0, 6, 2, 0, 2}, {1, 1, 1, 1, 1, 1, 1, 0}, {0, 2, 0, 2, 3, 1, 2, 3}};
    Case b = {"signed_range", 3, {1, 1, 2, 2, GRANQ_F32},
              {-1, 0.3f, 0.25f, 2.5f}, {-1}, {2.5f}, {0.5f}, {2},
              {-1, 0.5f, 0, 2.5f}, {1, 1, 1, 1}, {0, 3, 2, 7}};
    int failures = run(a, stream) + run(b, stream);
    HIP_OK(hipStreamDestroy(stream));
    if (failures) { std::printf("%d mismatches\n", failures); return 1; }
    std::printf("c_abi_client ok (%s)\n", granq_version());
    return 0;
}
