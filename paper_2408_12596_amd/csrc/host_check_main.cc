// Driver for a sanitizer build of the host-only part of the library (layout.cpp, analysis.cpp): reads one
// command per line from standard input, calls the C ABI, prints the results with full precision.  Built by
// `python -m paper_2408_12596_amd.build --host-sanitize` with AddressSanitizer and UndefinedBehaviorSanitizer on the
// host code; a CPU test feeds it the same cases it gives the library and compares the two outputs.
//   shard P N r
//   count arch L H nh F S V dtype
//   offset arch L H nh F S V dtype layer tensor
//   comm P world stage param_bytes grad_bytes bytes_per_second
//   curve mbs n b1 t1 ... bn tn
//   alloc stage gbs tcomm peak ndev { mbs n b1 t1 ... bn tn } x ndev
#include "../../include/poplar.h"
#include <cstdio>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

static poplar_model_cfg read_cfg(std::istream& in) {
  poplar_model_cfg c{};
  in >> c.arch >> c.n_layer >> c.hidden >> c.n_head >> c.ffn >> c.seq >> c.vocab >> c.dtype;
  c.world = 1; c.causal = 1;
  return c;
}

struct OwnedCurve {
  std::vector<int32_t> b;
  std::vector<double> t;
  poplar_curve c;
};
static void read_curve(std::istream& in, OwnedCurve& o) {
  int mbs = 0, n = 0;
  in >> mbs >> n;
  o.b.resize(n); o.t.resize(n);
  for (int i = 0; i < n; ++i) in >> o.b[i] >> o.t[i];
  o.c.n_pts = n; o.c.batch = o.b.data(); o.c.time = o.t.data(); o.c.mbs = mbs;
}

int main() {
  std::string line;
  while (std::getline(std::cin, line)) {
    std::istringstream in(line);
    std::string cmd;
    if (!(in >> cmd)) continue;
    int rc = 0;
    if (cmd == "shard") {
      int64_t P, off = 0, len = 0, valid = 0; int N, r;
      in >> P >> N >> r;
      rc = poplar_shard_range(P, N, r, &off, &len, &valid);
      std::printf("%d %lld %lld %lld\n", rc, (long long)off, (long long)len, (long long)valid);
    } else if (cmd == "count") {
      poplar_model_cfg c = read_cfg(in);
      int64_t pm = 0, pl = 0;
      rc = poplar_model_param_count(&c, &pm);
      if (rc == 0) rc = poplar_layer_param_count(&c, &pl);
      std::printf("%d %lld %lld\n", rc, (long long)pm, (long long)pl);
    } else if (cmd == "offset") {
      poplar_model_cfg c = read_cfg(in);
      int layer, tensor; int64_t off = 0, rows = 0, cols = 0;
      in >> layer >> tensor;
      rc = poplar_param_offset(&c, layer, tensor, &off, &rows, &cols);
      std::printf("%d %lld %lld %lld\n", rc, (long long)off, (long long)rows, (long long)cols);
    } else if (cmd == "comm") {
      int64_t P; int world, stage; double pb, gb, bw, o[5] = {0, 0, 0, 0, 0};
      in >> P >> world >> stage >> pb >> gb >> bw;
      rc = poplar_comm_model(P, world, stage, pb, gb, bw, &o[0], &o[1], &o[2], &o[3], &o[4]);
      std::printf("%d %.17g %.17g %.17g %.17g %.17g\n", rc, o[0], o[1], o[2], o[3], o[4]);
    } else if (cmd == "curve") {
      OwnedCurve oc;
      read_curve(in, oc);
      std::vector<double> sp(oc.c.mbs + 1, 0.0);
      rc = poplar_speed_curve(&oc.c, sp.data());
      std::printf("%d", rc);
      for (double v : sp) std::printf(" %.17g", v);
      std::printf("\n");
    } else if (cmd == "alloc") {
      int stage, ndev; long long gbs; double tc, peak;
      in >> stage >> gbs >> tc >> peak >> ndev;
      std::vector<OwnedCurve> oc(ndev);
      std::vector<poplar_curve> cs(ndev);
      for (int i = 0; i < ndev; ++i) { read_curve(in, oc[i]); cs[i] = oc[i].c; }
      std::vector<int32_t> g(ndev), b(ndev), ga(ndev), l(ndev);
      poplar_alloc out{g.data(), b.data(), ga.data(), l.data(), 0.0, 0.0, 0.0};
      rc = poplar_allocate(stage, ndev, cs.data(), gbs, tc, peak, &out);
      std::printf("%d", rc);
      if (rc == 0) {
        for (int i = 0; i < ndev; ++i) std::printf(" %d %d %d %d", g[i], b[i], ga[i], l[i]);
        std::printf(" %.17g %.17g %.17g", out.T, out.t, out.T_steps);
      } else {
        std::printf(" %s", poplar_last_error());
      }
      std::printf("\n");
    } else {
      std::printf("unknown command\n");
      return 2;
    }
  }
  return 0;
}
