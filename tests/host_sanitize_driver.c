/* Sweeps the host-only entry points of the library (parameter checks, workspace sizing, Eq. 7-8
 * utilities, error text handling) over the legal parameter range and its edges.  Built and linked
 * against a copy of the library whose host code carries AddressSanitizer and UndefinedBehaviorSanitizer;
 * any finding aborts the program.  No kernel is launched and no GPU is needed. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "asap.h"

static unsigned long long n_valid = 0, n_invalid = 0;
static size_t largest = 0;

static void probe(const asap_params* p) {
  char msg[160];
  asap_status st = asap_check_params(p, msg, sizeof(msg));
  size_t ws = asap_workspace_bytes(p), wa = asap_attention_workspace_bytes(p);
  if (st == ASAP_OK) {
    ++n_valid;
    if (ws == 0 || ws % 256 != 0) { printf("workspace of valid params: %zu\n", ws); exit(3); }
    if (ws > largest) largest = ws;
    (void)wa;
  } else {
    ++n_invalid;
    if (ws != 0 || wa != 0 || msg[0] == 0) { printf("invalid params gave a size or no message\n"); exit(4); }
  }
  /* short and missing message buffers */
  char tiny[4];
  (void)asap_check_params(p, tiny, sizeof(tiny));
  (void)asap_check_params(p, tiny, 1);
  (void)asap_check_params(p, tiny, 0);
  (void)asap_check_params(p, NULL, 0);
}

int main(void) {
  static const int Bs[] = {1, 2, 7, 16, 64, 2047}, Hs[] = {1, 4, 8, 28, 32, 40, 64}, Gs[] = {1, 2, 4, 7, 8},
                   ds[] = {64, 128}, Ds[] = {64, 256, 3584, 4096, 5120, 8192}, Ps[] = {0, 1, 35, 4096},
                   Vs[] = {1, 2, 31, 32, 33, 576, 1024, 1025, 2304, 4096, 16383, 16384},
                   Ts[] = {1, 2, 7, 28, 29, 31, 32, 33, 64, 65, 96, 97, 128};
  asap_params p;
  memset(&p, 0, sizeof(p));
  p.lambda_max = 1.0f; p.eps = 1e-6f; p.sim_threshold = -INFINITY; p.merge_weight = 1.0f;
  p.mask_mode = ASAP_MASK_KEYBIAS;
  for (unsigned ib = 0; ib < sizeof(Bs) / sizeof(*Bs); ++ib)
  for (unsigned ih = 0; ih < sizeof(Hs) / sizeof(*Hs); ++ih)
  for (unsigned ig = 0; ig < sizeof(Gs) / sizeof(*Gs); ++ig)
  for (unsigned id = 0; id < 2; ++id)
  for (unsigned iv = 0; iv < sizeof(Vs) / sizeof(*Vs); ++iv)
  for (unsigned it = 0; it < sizeof(Ts) / sizeof(*Ts); ++it) {
    p.B = Bs[ib]; p.H = Hs[ih]; p.Hkv = Hs[ih] % Gs[ig] == 0 ? Hs[ih] / Gs[ig] : Hs[ih];
    p.d = ds[id]; p.V = Vs[iv]; p.Tmax = Ts[it];
    p.D = Ds[(ib + ih + iv) % (sizeof(Ds) / sizeof(*Ds))];
    p.P = Ps[(ig + it) % (sizeof(Ps) / sizeof(*Ps))];
    const int ks[] = {1, p.V / 4 > 0 ? p.V / 4 : 1, p.V / 2 > 0 ? p.V / 2 : 1, p.V > 1 ? p.V - 1 : 1, p.V};
    for (unsigned ik = 0; ik < 5; ++ik)
    for (int dt = 0; dt < 2; ++dt)
    for (int route = 0; route < 2; ++route)
    for (int rows = 0; rows < 2; ++rows) {
      p.k = ks[ik];
      p.qk_dtype = p.h_dtype = (asap_dtype)dt;
      p.kv_dtype = (asap_dtype)((dt + ik) & 1);
      p.route = (asap_route)route;
      p.score_rows = (asap_score_rows)rows;
      probe(&p);
    }
  }
  /* edges and nonsense in every field: the checks must refuse, never compute with it */
  asap_params good;
  memset(&good, 0, sizeof(good));
  good.B = 16; good.H = 32; good.Hkv = 32; good.d = 128; good.D = 4096; good.P = 35; good.V = 2304; good.Tmax = 64;
  good.k = 320; good.qk_dtype = good.h_dtype = good.kv_dtype = ASAP_BF16;
  good.lambda_max = 1.0f; good.eps = 1e-6f; good.sim_threshold = -INFINITY; good.merge_weight = 1.0f;
  good.mask_mode = ASAP_MASK_KEYBIAS;
  static const int bad_ints[] = {-2147483647 - 1, -1, 0, 2147483647, 65536, 1 << 30};
  int32_t* fields[] = {&p.B, &p.H, &p.Hkv, &p.d, &p.D, &p.P, &p.V, &p.Tmax, &p.k};
  for (unsigned f = 0; f < sizeof(fields) / sizeof(*fields); ++f)
    for (unsigned v = 0; v < sizeof(bad_ints) / sizeof(*bad_ints); ++v) {
      p = good;
      *fields[f] = bad_ints[v];
      probe(&p);
    }
  static const float bad_floats[] = {NAN, INFINITY, -INFINITY, -1.0f, 0.0f, 1e38f};
  float* ffields[] = {&p.lambda_max, &p.eps, &p.sim_threshold, &p.merge_weight};
  for (unsigned f = 0; f < 4; ++f)
    for (unsigned v = 0; v < sizeof(bad_floats) / sizeof(*bad_floats); ++v) {
      p = good;
      *ffields[f] = bad_floats[v];
      probe(&p);
    }
  (void)asap_check_params(NULL, NULL, 0);
  if (asap_workspace_bytes(NULL) != 0) return 5;
  /* contexts without a GPU: creation fails cleanly, NULL contexts are tolerated where documented */
  asap_ctx* ctx = NULL;
  asap_status st = asap_create(&ctx, 0);
  if (st == ASAP_OK) asap_destroy(ctx);
  (void)asap_create(NULL, 0);
  (void)asap_create(&ctx, -1);
  asap_destroy(NULL);
  if (asap_last_error(NULL) == NULL) return 6;
  /* Eq. 7 / Eq. 8 utilities */
  {
    const int32_t layers[3] = {2, 14, 16}, tokens[3] = {2304, 576, 160};
    double f = 0.0, r = 0.0;
    if (asap_theoretical_flops(layers, tokens, 3, 5120, 13824, &f) != ASAP_OK || !(f > 0.0)) return 7;
    if (asap_flops_ratio(layers, tokens, 3, 2304, 5120, 13824, &r) != ASAP_OK || !(r > 0.0 && r < 1.0)) return 8;
    const int32_t big[1] = {2147483647};
    (void)asap_theoretical_flops(big, big, 1, 2147483647, 2147483647, &f);
    (void)asap_flops_ratio(big, big, 1, 2147483647, 2147483647, 2147483647, &r);
    const int32_t neg[1] = {-1};
    if (asap_theoretical_flops(neg, tokens, 1, 64, 64, &f) == ASAP_OK) return 9;
    if (asap_theoretical_flops(NULL, tokens, 1, 64, 64, &f) == ASAP_OK) return 10;
    if (asap_flops_ratio(layers, tokens, 0, 1, 1, 1, &r) == ASAP_OK) return 11;
  }
  printf("host sweep ok: %llu valid and %llu invalid parameter blocks, largest workspace %zu bytes\n", n_valid,
         n_invalid, largest);
  return 0;
}
