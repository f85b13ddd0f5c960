// Host-only driver for the sanitizer build of the library's host core (host.cpp, iter.cpp): walks the inference
// helpers, the descriptor checks and the operand iterator over a sweep of shapes, strides and dtypes.  No device call.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "common.h"
#include "iter.h"

using namespace tx;

static tx_tensor make(void* data, int dtype, std::vector<int64_t> sizes, std::vector<int64_t> strides) {
  tx_tensor t;
  memset(&t, 0, sizeof(t));
  t.data = data;
  t.dtype = dtype;
  t.ndim = (int)sizes.size();
  for (size_t i = 0; i < sizes.size(); ++i) { t.sizes[i] = sizes[i]; t.strides[i] = strides[i]; }
  return t;
}

int main() {
  static char buf[1 << 16];
  long calls = 0, errors = 0;
  const std::vector<std::vector<int64_t>> shapes = {{}, {1}, {5}, {0}, {3, 1}, {1, 4}, {3, 4}, {2, 3, 4}, {2, 1, 4, 1, 3, 1, 2, 2}, {0, 3}, {7, 1, 5}};
  auto contiguous = [](const std::vector<int64_t>& s) { std::vector<int64_t> st(s.size()); int64_t n = 1; for (int i = (int)s.size() - 1; i >= 0; --i) { st[i] = n; n *= s[i] > 0 ? s[i] : 1; } return st; };
  for (int da = 0; da <= 5; ++da)
    for (int db = 0; db <= 5; ++db)
      for (auto& sa : shapes)
        for (auto& sb : shapes) {
          tx_tensor a = make(buf, da, sa, contiguous(sa)), b = make(buf + 4096, db, sb, contiguous(sb));
          for (int op = 0; op < 8; ++op) {
            int32_t dt = -1, nd = -1;
            int64_t sizes[TX_MAX_DIMS];
            tx_status rc = tx_infer_binary(op, &a, &b, &dt, &nd, sizes);
            ++calls;
            if (rc) { ++errors; (void)tx_last_error(); (void)tx_strerror(rc); continue; }
            // the iterator on the inferred shape, output contiguous
            std::vector<int64_t> os(sizes, sizes + nd);
            tx_tensor out = make(buf + 8192, dt, os, contiguous(os));
            const tx_tensor* ops[3] = {&out, &a, &b};
            Iter it;
            iter_build(&it, nd, sizes, ops, 3);
            if (it.ndim < 1 || it.ndim > TX_MAX_DIMS) { printf("iterator rank %d\n", it.ndim); return 1; }
            const tx_tensor* ins[2] = {&a, &b};
            (void)check_out_overlap(&out, ins, 2);
          }
        }
  for (int dt = -1; dt <= 6; ++dt) {
    for (int op = -1; op < 64; ++op) { (void)tx_infer_unary_dtype(op, dt); ++calls; }
    for (int m = 0; m < 16; ++m) { (void)tx_infer_clamp_dtype(dt, m & 1, (m >> 1) & 1, (m >> 2) & 1, (m >> 3) & 1); ++calls; }
  }
  for (int da = 0; da <= 5; ++da)
    for (int db = 0; db <= 5; ++db)
      for (auto& sa : shapes) {
        tx_tensor a = make(buf, da, sa, contiguous(sa)), b = make(buf + 4096, db, {}, {});
        int32_t dt;
        errors += tx_infer_where(&a, &b, &dt) != 0;
        errors += tx_infer_where(&b, &a, &dt) != 0;
        calls += 2;
      }
  // overlap rules on views of one buffer
  for (int64_t off = 0; off < 24; off += 4)
    for (int64_t st = 0; st <= 2; ++st) {
      tx_tensor o = make(buf, TX_F32, {4, 3}, {3, 1}), v = make(buf + off, TX_F32, {4, 3}, {st * 3, st});
      errors += !no_internal_overlap(&v);
      errors += partial_overlap(&o, &v);
      calls += 2;
    }
  // descriptor checks on malformed input
  tx_tensor bad = make(buf, 9, {3}, {1});
  errors += check_tensor(&bad, "bad") != 0;
  bad = make(nullptr, TX_F32, {3}, {1});
  errors += check_tensor(&bad, "null data") != 0;
  bad = make(buf, TX_F32, {3, -1}, {1, 1});
  errors += check_tensor(&bad, "negative size") != 0;
  errors += check_tensor(nullptr, "null") != 0;
  tx_tensor wide = make(buf, TX_F32, {3}, {1});
  wide.ndim = 9;
  errors += check_tensor(&wide, "ndim") != 0;
  tx_force_path("generic");
  tx_force_path(nullptr);
  printf("host core: %ld calls, %ld refused, last path '%s'\n", calls, errors, tx_last_path());
  return 0;
}
