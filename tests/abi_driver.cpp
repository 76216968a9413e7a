// A caller of the C ABI that knows nothing of Python or PyTorch: device memory from hipMalloc,
// the default stream, files in and out.  The GPU test feeds it a seeded layer and compares what
// it writes with the CPU oracle.
//
//   abi_driver <dir>     reads <dir>/meta.txt, q.bin, K.bin, V.bin; writes scores.bin,
//                        budgets.bin, cu_seqlens.bin, indices.bin, K_out.bin, V_out.bin
// meta.txt: dtype h_q h_kv d w pool_k alpha flags batch, then batch values of n, then of B.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "adakv.h"

#define HIP_OK(x)                                                                      \
  do {                                                                                 \
    hipError_t e_ = (x);                                                               \
    if (e_ != hipSuccess) {                                                            \
      std::fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));              \
      return 2;                                                                        \
    }                                                                                  \
  } while (0)
#define ADAKV_OK_OR_DIE(x)                                                             \
  do {                                                                                 \
    int s_ = (x);                                                                      \
    if (s_ != ADAKV_OK) {                                                              \
      std::fprintf(stderr, "%s: %s\n", #x, adakv_strerror(s_));                        \
      return 3;                                                                        \
    }                                                                                  \
  } while (0)

static bool read_file(const std::string &path, std::vector<char> &buf) {
  FILE *f = std::fopen(path.c_str(), "rb");
  if (!f) return false;
  std::fseek(f, 0, SEEK_END);
  const long sz = std::ftell(f);
  std::fseek(f, 0, SEEK_SET);
  buf.resize((size_t)sz);
  const size_t got = sz ? std::fread(buf.data(), 1, (size_t)sz, f) : 0;
  std::fclose(f);
  return got == (size_t)sz;
}

static bool write_file(const std::string &path, const void *p, size_t bytes) {
  FILE *f = std::fopen(path.c_str(), "wb");
  if (!f) return false;
  const size_t put = bytes ? std::fwrite(p, 1, bytes, f) : 0;
  std::fclose(f);
  return put == bytes;
}

int main(int argc, char **argv) {
  if (argc != 2) {
    std::fprintf(stderr, "usage: abi_driver <dir>\n");
    return 1;
  }
  const std::string dir = argv[1];
  FILE *m = std::fopen((dir + "/meta.txt").c_str(), "r");
  if (!m) return 1;
  int dtype, h_q, h_kv, d, w, pool_k, batch;
  unsigned flags;
  float alpha;
  if (std::fscanf(m, "%d %d %d %d %d %d %f %u %d", &dtype, &h_q, &h_kv, &d, &w, &pool_k, &alpha,
                  &flags, &batch) != 9 || batch < 1 || batch > ADAKV_MAX_BATCH)
    return 1;
  std::vector<int32_t> n(batch), B(batch);
  std::vector<int64_t> tok_off(batch + 1, 0);
  for (int b = 0; b < batch; ++b) if (std::fscanf(m, "%d", &n[b]) != 1) return 1;
  for (int b = 0; b < batch; ++b) if (std::fscanf(m, "%d", &B[b]) != 1) return 1;
  std::fclose(m);
  long long scores_n = 0, rows_out = 0;
  for (int b = 0; b < batch; ++b) {
    tok_off[b + 1] = tok_off[b] + n[b] + w;
    scores_n += (long long)h_kv * n[b];
    rows_out += B[b];
  }
  const size_t esz = dtype == ADAKV_FP32 ? 4 : 2;
  const int nseg = batch * h_kv;

  adakv_layer L;
  L.dtype = dtype; L.h_q = h_q; L.h_kv = h_kv; L.d = d; L.w = w; L.pool_k = pool_k;
  L.alpha = alpha; L.scale = 0.0f; L.batch = batch;
  L.n = n.data(); L.B = B.data(); L.tok_off = tok_off.data();
  L.k_stride_tok = L.v_stride_tok = (int64_t)h_kv * d;
  L.k_stride_head = L.v_stride_head = d;
  L.flags = flags;

  std::vector<char> hq, hK, hV;
  if (!read_file(dir + "/q.bin", hq) || !read_file(dir + "/K.bin", hK) || !read_file(dir + "/V.bin", hV))
    return 1;
  if (hq.size() != (size_t)batch * h_q * w * d * esz || hK.size() != (size_t)tok_off[batch] * h_kv * d * esz ||
      hV.size() != hK.size()) {
    std::fprintf(stderr, "input sizes do not match meta.txt\n");
    return 1;
  }
  const size_t ws_bytes = adakv_workspace_bytes(&L);
  if (ws_bytes == 0) {
    std::fprintf(stderr, "layer rejected\n");
    return 3;
  }
  void *dq, *dK, *dV, *dws, *dKo, *dVo;
  float *dscores;
  int32_t *dbud, *dcu, *didx;
  HIP_OK(hipMalloc(&dq, hq.size()));
  HIP_OK(hipMalloc(&dK, hK.size()));
  HIP_OK(hipMalloc(&dV, hV.size()));
  HIP_OK(hipMalloc(&dws, ws_bytes));
  HIP_OK(hipMalloc((void **)&dscores, (size_t)scores_n * 4));
  HIP_OK(hipMalloc((void **)&dbud, (size_t)nseg * 4));
  HIP_OK(hipMalloc((void **)&dcu, (size_t)(nseg + 1) * 4));
  HIP_OK(hipMalloc((void **)&didx, (size_t)rows_out * 4));
  HIP_OK(hipMalloc(&dKo, (size_t)rows_out * d * esz));
  HIP_OK(hipMalloc(&dVo, (size_t)rows_out * d * esz));
  HIP_OK(hipMemcpy(dq, hq.data(), hq.size(), hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dK, hK.data(), hK.size(), hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dV, hV.data(), hV.size(), hipMemcpyHostToDevice));

  ADAKV_OK_OR_DIE(adakv_score(&L, dq, dK, nullptr, dscores, dws, ws_bytes, nullptr));
  ADAKV_OK_OR_DIE(adakv_allocate(&L, dscores, dbud, dcu, dws, ws_bytes, nullptr));
  ADAKV_OK_OR_DIE(adakv_select(&L, dscores, dbud, dcu, didx, dws, ws_bytes, nullptr));
  ADAKV_OK_OR_DIE(adakv_compact(&L, dK, dV, didx, dcu, dKo, dVo, nullptr));
  HIP_OK(hipDeviceSynchronize());

  std::vector<char> out;
  auto dump = [&](const char *name, const void *dev, size_t bytes) -> bool {
    out.resize(bytes);
    if (bytes && hipMemcpy(out.data(), dev, bytes, hipMemcpyDeviceToHost) != hipSuccess) return false;
    return write_file(dir + "/" + name, out.data(), bytes);
  };
  const bool ok = dump("scores.bin", dscores, (size_t)scores_n * 4) && dump("budgets.bin", dbud, (size_t)nseg * 4) &&
                  dump("cu_seqlens.bin", dcu, (size_t)(nseg + 1) * 4) && dump("indices.bin", didx, (size_t)rows_out * 4) &&
                  dump("K_out.bin", dKo, (size_t)rows_out * d * esz) && dump("V_out.bin", dVo, (size_t)rows_out * d * esz);
  for (void *p : {dq, dK, dV, dws, (void *)dscores, (void *)dbud, (void *)dcu, (void *)didx, dKo, dVo}) (void)hipFree(p);
  std::printf("abi_driver: %d sequence(s), %lld scores, %lld rows kept\n", batch, scores_n, rows_out);
  return ok ? 0 : 2;
}
