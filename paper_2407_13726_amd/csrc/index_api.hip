// Host entry points of the index-polynomial module (declared in dastac.h).
// Pure functions; no device is touched.
#include "common.h"

using namespace dastac;

extern "C" {

const char *dastac_strerror(int status) {
  switch (status) {
    case DASTAC_OK: return "ok";
    case DASTAC_EINVAL: return "invalid argument";
    case DASTAC_ENULL: return "null pointer";
    case DASTAC_EOVERFLOW: return "element count overflows the guarded 64-bit range";
    case DASTAC_EALIAS: return "output overlaps an input";
    case DASTAC_EHIP: return "HIP runtime error at launch";
    default: return "unknown status";
  }
}

int64_t dastac_tri_count(int64_t n) {
  if (n < 0 || n > DASTAC_TRI_MAX_N) return -1;
  return tri(n);
}

int64_t dastac_tet_count(int64_t n) {
  if (n < 0 || n > DASTAC_TET_MAX_N) return -1;
  return tet(n);
}

int64_t dastac_band_count(int64_t n, int64_t w) {
  if (n < 0 || w < 0 || w > (1LL << 30)) return -1;
  int64_t diags = 2 * w + 1;
  if (n != 0 && diags > ((int64_t)1 << 62) / n) return -1;
  return diags * n;
}

int64_t dastac_tri_offset(int64_t n, int64_t i, int64_t j) {
  if (n < 0 || n > DASTAC_TRI_MAX_N || i < 0 || j < i || j >= n) return -1;
  return tri_offset(n, i, j);
}

int64_t dastac_tril_offset(int64_t n, int64_t i, int64_t j) {
  if (n < 0 || n > DASTAC_TRI_MAX_N || j < 0 || i < j || i >= n) return -1;
  return (i * (i + 1)) / 2 + j;
}

int64_t dastac_tet_offset(int64_t n, int64_t i, int64_t j, int64_t k) {
  if (n < 0 || n > DASTAC_TET_MAX_N || i < 0 || j < i || k < j || k >= n) return -1;
  return tet_offset(n, i, j, k);
}

int64_t dastac_band_offset(int64_t n, int64_t w, int64_t d, int64_t i) {
  if (dastac_band_count(n, w) < 0 || d < -w || d > w || i < 0 || i >= n) return -1;
  return band_offset(n, w, d, i);
}

int dastac_tri_inverse(int64_t n, int64_t p, int64_t *i, int64_t *j) {
  if (!i || !j) return DASTAC_ENULL;
  if (n < 0 || n > DASTAC_TRI_MAX_N || p < 0 || p >= tri(n)) return DASTAC_EINVAL;
  tri_inverse(n, p, *i, *j);
  return DASTAC_OK;
}

int dastac_tet_inverse(int64_t n, int64_t p, int64_t *i, int64_t *j, int64_t *k) {
  if (!i || !j || !k) return DASTAC_ENULL;
  if (n < 0 || n > DASTAC_TET_MAX_N || p < 0 || p >= tet(n)) return DASTAC_EINVAL;
  tet_inverse(n, p, *i, *j, *k);
  return DASTAC_OK;
}

}  // extern "C"
