/* A client of libinfinipot written against the C header alone: no Python, no torch.  It fills a small pot with
 * pseudo-random bf16 data, calls ccd_compress through the C ABI and checks on the host what can be checked without
 * an oracle: the return codes, k strictly ascending indices per unit, every NuC slot kept, and K', V' being bit copies
 * of the rows the indices name; then it fills the pot up again with ccd_append and checks the rows.  Prints
 * "ccd_client ok" and exits 0 on success. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "infinipot.h"

#define CHECK_HIP(x)                                                                   \
  do {                                                                                 \
    hipError_t e_ = (x);                                                               \
    if (e_ != hipSuccess) {                                                            \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
      return 2;                                                                        \
    }                                                                                  \
  } while (0)

static uint32_t rng_state = 12345u;
static uint32_t next_u32(void) {
  rng_state = rng_state * 1664525u + 1013904223u;
  return rng_state;
}
/* roughly N(0,1) as a sum of uniforms, stored as bf16 bits (truncation is fine for test data) */
static uint16_t next_bf16(void) {
  float s = 0.f;
  for (int i = 0; i < 6; ++i) s += (float)(next_u32() >> 8) / 16777216.0f;
  s = (s - 3.0f) * 1.4142f;
  uint32_t bits;
  memcpy(&bits, &s, 4);
  return (uint16_t)(bits >> 16);
}

int main(void) {
  enum { B = 1, L = 2, HQ = 8, HKV = 2, D = 128, N = 640, K_KEEP = 256, P = 8, T = 64 };
  const size_t kv_elems = (size_t)B * L * HKV * N * D, q_elems = (size_t)B * L * HQ * P * D;
  uint16_t* hK = malloc(kv_elems * 2);
  uint16_t* hV = malloc(kv_elems * 2);
  uint16_t* hQ = malloc(q_elems * 2);
  float* hnov = malloc(sizeof(float) * B * N);
  if (!hK || !hV || !hQ || !hnov) return 2;
  for (size_t i = 0; i < kv_elems; ++i) { hK[i] = next_bf16(); hV[i] = next_bf16(); }
  for (size_t i = 0; i < q_elems; ++i) hQ[i] = next_bf16();
  for (int i = 0; i < B * N; ++i) hnov[i] = (float)(next_u32() >> 8) / 16777216.0f;

  ccd_shape_t s;
  memset(&s, 0, sizeof s);
  s.B = B; s.L = L; s.Hq = HQ; s.Hkv = HKV; s.d = D; s.n_valid = N; s.n_cap = N; s.k = K_KEEP; s.P = P; s.T = T;
  s.pool_w = 7; s.pool_mode = CCD_POOL_MAX; s.dtype = CCD_BF16; s.scale = 0.f;
  s.kv_stride_h = (int64_t)N * D; s.kv_stride_l = (int64_t)HKV * N * D; s.kv_stride_b = (int64_t)L * HKV * N * D;
  s.q_stride_h = (int64_t)P * D; s.q_stride_l = (int64_t)HQ * P * D; s.q_stride_b = (int64_t)L * HQ * P * D;
  s.nov_stride_b = N;

  const size_t ws_bytes = ccd_workspace_bytes(&s);
  if (ws_bytes == 0) { fprintf(stderr, "workspace size 0\n"); return 1; }
  void *dK, *dV, *dQ, *dws;
  float* dnov;
  int32_t* dkeep;
  CHECK_HIP(hipMalloc(&dK, kv_elems * 2));
  CHECK_HIP(hipMalloc(&dV, kv_elems * 2));
  CHECK_HIP(hipMalloc(&dQ, q_elems * 2));
  CHECK_HIP(hipMalloc((void**)&dnov, sizeof(float) * B * N));
  CHECK_HIP(hipMalloc((void**)&dkeep, sizeof(int32_t) * B * L * HKV * K_KEEP));
  CHECK_HIP(hipMalloc(&dws, ws_bytes));
  CHECK_HIP(hipMemcpy(dK, hK, kv_elems * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dV, hV, kv_elems * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dQ, hQ, q_elems * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dnov, hnov, sizeof(float) * B * N, hipMemcpyHostToDevice));

  /* a pot that is not full is left alone */
  ccd_shape_t not_full = s;
  not_full.n_valid = N - 1;
  int rc = ccd_compress(&not_full, dQ, dK, dV, dnov, NULL, dkeep, dws, ws_bytes, NULL);
  if (rc != CCD_NOOP) { fprintf(stderr, "expected CCD_NOOP, got %d (%s)\n", rc, ccd_strerror(rc)); return 1; }
  /* a workspace that is too small is refused on the host */
  rc = ccd_compress(&s, dQ, dK, dV, dnov, NULL, dkeep, dws, ws_bytes - 1, NULL);
  if (rc != CCD_EWORKSPACE) { fprintf(stderr, "expected CCD_EWORKSPACE, got %d\n", rc); return 1; }

  rc = ccd_compress(&s, dQ, dK, dV, dnov, NULL, dkeep, dws, ws_bytes, NULL);
  if (rc != CCD_OK) { fprintf(stderr, "ccd_compress: %d (%s)\n", rc, ccd_strerror(rc)); return 1; }
  CHECK_HIP(hipDeviceSynchronize());

  int32_t* keep = malloc(sizeof(int32_t) * B * L * HKV * K_KEEP);
  uint16_t* oK = malloc(kv_elems * 2);
  uint16_t* oV = malloc(kv_elems * 2);
  if (!keep || !oK || !oV) return 2;
  CHECK_HIP(hipMemcpy(keep, dkeep, sizeof(int32_t) * B * L * HKV * K_KEEP, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(oK, dK, kv_elems * 2, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(oV, dV, kv_elems * 2, hipMemcpyDeviceToHost));

  /* the T most novel tokens (ties cannot occur in this data with any likelihood worth handling) */
  char is_nuc[N];
  memset(is_nuc, 0, sizeof is_nuc);
  for (int t = 0; t < N; ++t) {
    int larger = 0;
    for (int j = 0; j < N; ++j) larger += hnov[j] > hnov[t] || (hnov[j] == hnov[t] && j < t);
    is_nuc[t] = larger < T;
  }
  for (int u = 0; u < B * L * HKV; ++u) {
    const int32_t* ku = keep + (size_t)u * K_KEEP;
    int nuc_kept = 0;
    for (int j = 0; j < K_KEEP; ++j) {
      if (ku[j] < 0 || ku[j] >= N || (j > 0 && ku[j] <= ku[j - 1])) { fprintf(stderr, "unit %d: keep_idx not ascending in range\n", u); return 1; }
      nuc_kept += is_nuc[ku[j]];
      const size_t src = ((size_t)u * N + (size_t)ku[j]) * D, dst = ((size_t)u * N + (size_t)j) * D;
      if (memcmp(oK + dst, hK + src, D * 2) != 0 || memcmp(oV + dst, hV + src, D * 2) != 0) {
        fprintf(stderr, "unit %d row %d is not a bit copy of row %d\n", u, j, ku[j]);
        return 1;
      }
    }
    if (nuc_kept != T) { fprintf(stderr, "unit %d keeps %d of the %d NuC slots\n", u, nuc_kept, T); return 1; }
  }
  /* the pot is filled up again behind the kept tokens (Sec. 3.2): N - K_KEEP new rows per unit */
  enum { M = N - K_KEEP };
  const size_t chunk_elems = (size_t)B * L * HKV * M * D;
  uint16_t* cK = malloc(chunk_elems * 2);
  uint16_t* cV = malloc(chunk_elems * 2);
  if (!cK || !cV) return 2;
  for (size_t i = 0; i < chunk_elems; ++i) { cK[i] = next_bf16(); cV[i] = next_bf16(); }
  void *dcK, *dcV;
  CHECK_HIP(hipMalloc(&dcK, chunk_elems * 2));
  CHECK_HIP(hipMalloc(&dcV, chunk_elems * 2));
  CHECK_HIP(hipMemcpy(dcK, cK, chunk_elems * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dcV, cV, chunk_elems * 2, hipMemcpyHostToDevice));
  ccd_shape_t after = s;
  after.n_valid = K_KEEP;
  rc = ccd_append(&after, dK, dV, NULL, dcK, dcV, NULL, M + 1, NULL);
  if (rc != CCD_EINVAL) { fprintf(stderr, "a chunk that does not fit: expected CCD_EINVAL, got %d\n", rc); return 1; }
  rc = ccd_append(&after, dK, dV, NULL, dcK, dcV, NULL, M, NULL);
  if (rc != CCD_OK) { fprintf(stderr, "ccd_append: %d (%s)\n", rc, ccd_strerror(rc)); return 1; }
  CHECK_HIP(hipDeviceSynchronize());
  uint16_t* aK = malloc(kv_elems * 2);
  uint16_t* aV = malloc(kv_elems * 2);
  if (!aK || !aV) return 2;
  CHECK_HIP(hipMemcpy(aK, dK, kv_elems * 2, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(aV, dV, kv_elems * 2, hipMemcpyDeviceToHost));
  for (int u = 0; u < B * L * HKV; ++u) {
    const size_t head = (size_t)u * N * D, kept = (size_t)K_KEEP * D, fresh = (size_t)M * D;
    if (memcmp(aK + head, oK + head, kept * 2) != 0 || memcmp(aV + head, oV + head, kept * 2) != 0) {
      fprintf(stderr, "unit %d: the append touched the kept rows\n", u);
      return 1;
    }
    if (memcmp(aK + head + kept, cK + (size_t)u * fresh, fresh * 2) != 0 ||
        memcmp(aV + head + kept, cV + (size_t)u * fresh, fresh * 2) != 0) {
      fprintf(stderr, "unit %d: the appended rows are not bit copies of the chunk\n", u);
      return 1;
    }
  }
  printf("ccd_client ok: %d units, %d -> %d tokens, %d appended\n", B * L * HKV, N, K_KEEP, M);
  return 0;
}
