// Host-only driver for a sanitizer build of the library (address + undefined-behaviour sanitizers on the HOST code;
// device code is compiled as usual and never runs here).  It walks the argument-validation and planning paths of the
// C-ABI that touch no device: every call below must return the documented code, and the sanitizers must stay silent.
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "../include/dn.h"

#define EXPECT(expr, want)                                                                     \
    do {                                                                                       \
        const long long got_ = (long long)(expr);                                              \
        if (got_ != (long long)(want)) {                                                       \
            std::printf("FAIL %s:%d: %s = %lld, expected %lld\n", __FILE__, __LINE__, #expr, got_, (long long)(want)); \
            return 1;                                                                          \
        }                                                                                      \
    } while (0)

int main() {
    // creation: valid and invalid networks, the largest layer count, sizes
    const int dims_a[] = {784, 300, 300, 10};
    dn_ctx* a = nullptr;
    EXPECT(dn_create(&a, 3, dims_a, 60000.0, 60000, 3000), DN_OK);
    EXPECT(dn_num_params(a), 328810);
    EXPECT(dn_workspace_bytes(a) > 4ull * 3000 * 10 * 600, 1);
    EXPECT(dn_num_partitions(a), 0);
    std::vector<int> deep(11, 5);
    dn_ctx* b = nullptr;
    EXPECT(dn_create(&b, 8, deep.data(), 1.0, 7, 3), DN_OK);          // DN_MAX_LAYERS weight layers
    dn_ctx* c = reinterpret_cast<dn_ctx*>(0x10);
    EXPECT(dn_create(&c, 9, deep.data(), 1.0, 7, 3), DN_EINVAL);      // one more: refused, the handle reset to null
    EXPECT(c == nullptr, 1);
    const int bad[] = {4, 0, 2};
    EXPECT(dn_create(&c, 2, bad, 1.0, 1, 1), DN_EINVAL);
    EXPECT(dn_create(nullptr, 2, dims_a, 1.0, 1, 1), DN_EINVAL);
    EXPECT(dn_create(&c, 3, dims_a, -1.0, 1, 1), DN_EINVAL);
    // slice plans of the sums over samples for every subsample size (the planner's table walks)
    for (int s = 1; s <= 3000; ++s)
        if (dn_product_slices(a, s) < 1) { std::printf("FAIL: no plan for s = %d\n", s); return 1; }
    EXPECT(dn_product_slices(a, 3001), DN_EINVAL);
    // call order: nothing bound yet
    float* fake = reinterpret_cast<float*>(0x1000);      // never dereferenced: validation fails first
    double f = 0.0;
    int it = 0;
    EXPECT(dn_forward(a, fake, fake, fake, 10, &f, nullptr), DN_ESTATE);
    EXPECT(dn_grad(a, fake, fake, fake, 10, fake, nullptr), DN_ESTATE);
    EXPECT(dn_gn_matvec(a, fake, fake, DN_FULL), DN_ESTATE);
    EXPECT(dn_bind(a, nullptr, 1 << 20, nullptr), DN_EINVAL);
    EXPECT(dn_bind(a, reinterpret_cast<void*>(0x1001), 1 << 20, nullptr), DN_EINVAL);
    EXPECT(dn_bind(a, fake, 16, nullptr), DN_ENOSPC);
    EXPECT(dn_bind(a, fake, dn_workspace_bytes(a), nullptr), DN_OK);
    EXPECT(dn_forward(a, nullptr, fake, fake, 10, &f, nullptr), DN_EINVAL);
    EXPECT(dn_jacobian_prep(a, fake, fake, 100, reinterpret_cast<const int*>(fake), 3001), DN_EINVAL);
    EXPECT(dn_gn_matvec(a, fake, fake, 7), DN_EINVAL);
    EXPECT(dn_gn_matvec(a, fake, fake, DN_PARTITION), DN_ESTATE);
    EXPECT(dn_cg(a, fake, 1.0, 0.0, 5, DN_FULL, fake, &it, &f), DN_ESTATE);
    EXPECT(dn_cg(a, fake, -1.0, 0.0, 5, DN_FULL, fake, &it, &f), DN_EINVAL);
    EXPECT(dn_cg_sync(a, fake, 1.0, 1e-3, 5, DN_FULL, 0, 50.0, fake, &it, &f), DN_EINVAL);
    const int too_many[] = {1, 5, 1, 1};
    EXPECT(dn_set_split(a, too_many), DN_EINVAL);
    EXPECT(dn_set_split(a, nullptr), DN_EINVAL);
    EXPECT(dn_jacobian_read(a, 3, fake), DN_EINVAL);
    EXPECT(dn_jacobian_read(a, 1, fake), DN_ESTATE);
    dn_newton_params prm = {1.0, 1e-3, 1e-4, 1e-5, 2.0 / 3.0, 1.5, 10, DN_FULL, 1, 30, 0, 0.0, 0};
    dn_newton_stats st;
    EXPECT(dn_newton_step(a, fake, fake, fake, 10, reinterpret_cast<const int*>(fake), 3001, fake, &prm, &st), DN_EINVAL);
    prm.eta = 1.0;
    EXPECT(dn_newton_step(a, fake, fake, fake, 10, reinterpret_cast<const int*>(fake), 5, fake, &prm, &st), DN_EINVAL);
    EXPECT(dn_set_stream_passes(a, 1), DN_EINVAL);
    EXPECT(dn_set_stream_passes(a, 2), DN_OK);
    EXPECT(dn_set_spin_limit(a, 0), DN_OK);
    // the entry point without a context
    EXPECT(dn_forward_static(3, dims_a, 1.0, fake, fake, fake, 20000, nullptr, &f, nullptr), DN_ETOOBIG);
    EXPECT(dn_forward_static(3, dims_a, 1.0, fake, fake, fake, 0, nullptr, &f, nullptr), DN_EINVAL);
    EXPECT(dn_forward_static(9, deep.data(), 1.0, fake, fake, fake, 5, nullptr, &f, nullptr), DN_EINVAL);
    // profile bookkeeping without a device
    EXPECT(dn_profile_num_classes() >= 10, 1);
    EXPECT(dn_profile_class_name(-1) == nullptr, 1);
    EXPECT(dn_profile_class_name(dn_profile_num_classes()) == nullptr, 1);
    EXPECT(dn_strerror(DN_ETOOBIG) != nullptr, 1);
    EXPECT(dn_strerror(12345) != nullptr, 1);
    dn_destroy(a);
    dn_destroy(b);
    dn_destroy(nullptr);
    std::printf("host driver ok\n");
    return 0;
}
