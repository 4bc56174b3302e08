// host-only sanitizer run of the plan builder and the bucketing programme (random tables)
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "plan.h"
extern "C" lobra_status lobra_dynamic_buckets(const int32_t*, int64_t, const int32_t*, int32_t, int32_t, int32_t*, int32_t*, int64_t*);
int main() {
  std::mt19937 rng(7);
  for (int it = 0; it < 3000; ++it) {
    int S = rng() % 40, n = rng() % 6;
    std::vector<int32_t> off(1, 0), task, ro(1, 0);
    // every third table describes fused shared-input projections: ranks and width multiples of 8 P
    const int P = it % 3 == 2 ? 2 + int(rng() % 3) : 1;
    for (int t = 0; t < n; ++t) ro.push_back(ro.back() + (P > 1 ? 8 * P * (1 + int(rng() % (16 / P))) : 1 + int(rng() % 128)));
    static const int L[] = {0, 1, 2, 15, 16, 17, 31, 32, 33, 64, 100, 255, 256, 257, 1000};
    for (int k = 0; k < S; ++k) { off.push_back(off.back() + L[rng() % 15]); task.push_back(int(rng() % (n + 1)) - 1); }
    lobra_mlora_desc d{};
    d.dtype = rng() % 2; d.d_in = 8 * (1 + rng() % 600); d.d_out = 8 * (1 + rng() % 600); d.T = off.back(); d.n_tasks = n; d.S = S;
    d.rank_off = ro.data(); d.seg_off = off.data(); d.seg_task = task.data();
    if (P > 1) { d.n_proj = P; d.d_out = 8 * P * (1 + rng() % 100); }
    if (S == 0) d.T = 0;
    lobra_status st = lobra::validate(&d);
    if (st != LOBRA_OK) { printf("validate %d at it %d\n", st, it); return 1; }
    lobra::Plan p;
    st = lobra::build_host_plan(&d, rng() % 4, &p);
    if (st != LOBRA_OK) { printf("plan %d\n", st); return 1; }
    auto blob = lobra::pack_blob(&p);
    (void)blob;
    // bucketing
    int U = 1 + rng() % 64, R = 1 + rng() % 20;
    std::vector<int32_t> u; int32_t b = 0; for (int i = 0; i < U; ++i) { b += 1 + rng() % 300; u.push_back(b); }
    std::vector<int32_t> lens; int ns = rng() % 200; for (int i = 0; i < ns; ++i) lens.push_back(1 + rng() % u.back());
    std::vector<int32_t> ob(R); int32_t on = 0; int64_t pad = 0;
    st = lobra_dynamic_buckets(lens.data(), ns, u.data(), U, R, ob.data(), &on, &pad);
    if (st != LOBRA_OK || on > R) { printf("bucket %d\n", st); return 1; }
  }
  printf("host fuzz ok\n");
  return 0;
}
