// Host-side entry points of the cost model (Sec. 3.2.3, App. A): the expected expert union under
// uniform routing, the least-squares cost surface over (verification length, union), its collapse to
// the table C(k) that prefix selection divides by, and a text file format for that table. Init-time
// logic on a few hundred profiling points; nothing here touches the GPU.
#include <errno.h>
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "common.h"

using namespace evict;

namespace {

// App. A: M (1 - (1 - K/M)^t)
double union_closed_form(int M, int K, double t) { return M * (1.0 - pow(1.0 - (double)K / M, t)); }

const char kTableMagic[] = "evict-cost-table";

bool key_ok(const char* key) {
  if (!key) return false;
  const size_t n = strlen(key);
  if (n < 1 || n > 255) return false;
  for (size_t i = 0; i < n; ++i)
    if (key[i] <= ' ' || key[i] > '~') return false;
  return true;
}

}  // namespace

extern "C" {

int evict_cost_expected_union_host(int n_experts, int top_k, const double* t, int n, double* out) {
  EVICT_REQUIRE(n_experts >= 1 && top_k >= 1 && top_k <= n_experts, EVICT_E_INVALID,
                "evict_cost_expected_union_host: need 1 <= top_k <= n_experts (got %d, %d)", top_k, n_experts);
  EVICT_REQUIRE(n >= 0 && (n == 0 || (t && out)), EVICT_E_INVALID, "evict_cost_expected_union_host: null array");
  for (int i = 0; i < n; ++i) {
    EVICT_REQUIRE(t[i] >= 0.0, EVICT_E_INVALID, "evict_cost_expected_union_host: t[%d] = %g is negative", i, t[i]);
    out[i] = union_closed_form(n_experts, top_k, t[i]);
  }
  return EVICT_OK;
}

int evict_cost_fit_surface_host(const double* k, const double* u, const double* ms, int n, double* coef, double* rms) {
  EVICT_REQUIRE(k && u && ms && coef, EVICT_E_INVALID, "evict_cost_fit_surface_host: null array");
  EVICT_REQUIRE(n >= 3, EVICT_E_INVALID, "evict_cost_fit_surface_host: need at least 3 points (got %d)", n);
  // ms ~ a + b k + c U by least squares. The columns are centred first, which leaves a 2 x 2 system
  // in (b, c) whose determinant says whether the points span the (k, U) plane.
  double kb = 0, ub = 0, mb = 0;
  for (int i = 0; i < n; ++i) { kb += k[i]; ub += u[i]; mb += ms[i]; }
  kb /= n; ub /= n; mb /= n;
  double skk = 0, suu = 0, sku = 0, skm = 0, sum = 0;
  for (int i = 0; i < n; ++i) {
    const double dk = k[i] - kb, du = u[i] - ub, dm = ms[i] - mb;
    skk += dk * dk; suu += du * du; sku += dk * du; skm += dk * dm; sum += du * dm;
  }
  const double det = skk * suu - sku * sku;
  EVICT_REQUIRE(skk > 0 && suu > 0 && det > 1e-10 * skk * suu, EVICT_E_INVALID,
                "evict_cost_fit_surface_host: the (k, union) points lie on one line; profile inputs of another routing spread");
  const double b = (skm * suu - sum * sku) / det;
  const double c = (sum * skk - skm * sku) / det;
  const double a = mb - b * kb - c * ub;
  coef[0] = a; coef[1] = b; coef[2] = c;
  if (rms) {
    double ss = 0;
    for (int i = 0; i < n; ++i) { const double r = a + b * k[i] + c * u[i] - ms[i]; ss += r * r; }
    *rms = sqrt(ss / n);
  }
  return EVICT_OK;
}

int evict_cost_collapse_host(const double* coef, int k_max, int n_experts, int top_k, const double* union_of_k,
                             int n_union, float* cost) {
  EVICT_REQUIRE(coef && cost, EVICT_E_INVALID, "evict_cost_collapse_host: null array");
  EVICT_REQUIRE(k_max >= 0, EVICT_E_INVALID, "evict_cost_collapse_host: k_max = %d", k_max);
  EVICT_REQUIRE(n_experts >= 1 && top_k >= 1 && top_k <= n_experts, EVICT_E_INVALID,
                "evict_cost_collapse_host: need 1 <= top_k <= n_experts (got %d, %d)", top_k, n_experts);
  EVICT_REQUIRE(n_union >= 0 && (n_union == 0 || union_of_k), EVICT_E_INVALID, "evict_cost_collapse_host: null union_of_k");
  std::vector<double> c((size_t)k_max + 1);
  for (int kk = 0; kk <= k_max; ++kk) {
    // the union measured at this length where there is one, the closed form otherwise
    double un = union_closed_form(n_experts, top_k, (double)kk);
    if (kk < n_union && union_of_k[kk] > 0.0) un = union_of_k[kk];
    c[kk] = coef[0] + coef[1] * kk + coef[2] * un;
  }
  if (k_max >= 1) c[0] = c[1];  // no prefix is empty: entry 0 repeats entry 1
  for (int kk = 0; kk <= k_max; ++kk)
    EVICT_REQUIRE(c[kk] > 0.0 && isfinite(c[kk]), EVICT_E_INVALID,
                  "evict_cost_collapse_host: the fitted surface is not positive over the table's range (C(%d) = %g)", kk, c[kk]);
  for (int kk = 0; kk <= k_max; ++kk) cost[kk] = (float)c[kk];
  return EVICT_OK;
}

int evict_cost_table_save_host(const char* path, const float* cost, int k_max, const char* key) {
  EVICT_REQUIRE(path && cost && k_max >= 0, EVICT_E_INVALID, "evict_cost_table_save_host: bad argument");
  EVICT_REQUIRE(key_ok(key), EVICT_E_INVALID, "evict_cost_table_save_host: the key must be 1..255 printable characters without white space");
  for (int kk = 0; kk <= k_max; ++kk)
    EVICT_REQUIRE(cost[kk] > 0.0f && isfinite(cost[kk]), EVICT_E_INVALID, "evict_cost_table_save_host: C(%d) = %g is not a positive number", kk, (double)cost[kk]);
  FILE* f = fopen(path, "w");
  EVICT_REQUIRE(f, EVICT_E_INVALID, "evict_cost_table_save_host: cannot open %s: %s", path, strerror(errno));
  bool ok = fprintf(f, "%s 1 %d %s\n", kTableMagic, k_max, key) > 0;
  for (int kk = 0; ok && kk <= k_max; ++kk) ok = fprintf(f, "%.9g\n", (double)cost[kk]) > 0;  // 9 digits: a float survives the round trip
  ok = (fclose(f) == 0) && ok;
  EVICT_REQUIRE(ok, EVICT_E_INVALID, "evict_cost_table_save_host: write to %s failed", path);
  return EVICT_OK;
}

int evict_cost_table_load_host(const char* path, const char* expect_key, float* cost, int capacity, int* k_max) {
  EVICT_REQUIRE(path && k_max, EVICT_E_INVALID, "evict_cost_table_load_host: bad argument");
  FILE* f = fopen(path, "r");
  EVICT_REQUIRE(f, EVICT_E_INVALID, "evict_cost_table_load_host: cannot open %s: %s", path, strerror(errno));
  char magic[32] = {0}, key[256] = {0};
  int version = 0, km = -1;
  const bool head = fscanf(f, "%31s %d %d %255s", magic, &version, &km, key) == 4 && !strcmp(magic, kTableMagic) && version == 1 && km >= 0;
  if (!head) {
    fclose(f);
    set_error("evict_cost_table_load_host: %s is not a cost table of format 1", path);
    return EVICT_E_INVALID;
  }
  if (expect_key && strcmp(expect_key, key)) {
    fclose(f);
    set_error("evict_cost_table_load_host: %s was profiled for \"%s\", not for \"%s\"", path, key, expect_key);
    return EVICT_E_INVALID;
  }
  *k_max = km;
  if (!cost) { fclose(f); return EVICT_OK; }  // size query
  if (capacity < km + 1) {
    fclose(f);
    set_error("evict_cost_table_load_host: the table has %d entries, the buffer %d", km + 1, capacity);
    return EVICT_E_INVALID;
  }
  for (int kk = 0; kk <= km; ++kk) {
    float v;
    if (fscanf(f, "%f", &v) != 1 || !(v > 0.0f) || !isfinite(v)) {
      fclose(f);
      set_error("evict_cost_table_load_host: entry %d of %s is missing or not a positive number", kk, path);
      return EVICT_E_INVALID;
    }
    cost[kk] = v;
  }
  fclose(f);
  return EVICT_OK;
}

}  // extern "C"
