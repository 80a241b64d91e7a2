// Definitions behind the tuning hook; empty unless the library is built with -DPF_TUNING (see tuning.h).
#include "tuning.h"

#include "ops.h"

#ifdef PF_TUNING
namespace pf {
int g_attn_variant = 0, g_attn_stages = 0, g_attn_wide = 0, g_force_splits = 0, g_fuse_kv_route = 1, g_fold_q_scale = 1;
int g_gemm_tile_override = 0, g_wavek_min_k = 2048, g_wavek_max_tiles = 512;
}  // namespace pf

extern "C" void pf_tune(int id) {
  using namespace pf;
  if (id >= 800) g_fold_q_scale = id - 800;
  else if (id >= 700) g_attn_wide = id - 700;
  else if (id >= 600) g_force_splits = id - 600;
  else if (id >= 500) g_wavek_max_tiles = (id - 500) * 16;
  else if (id >= 400) g_wavek_min_k = (id - 400) * 64;
  else if (id >= 300) g_attn_stages = id - 300;
  else if (id >= 200) g_fuse_kv_route = id - 200;
  else if (id >= 100) g_attn_variant = id - 100;
  else g_gemm_tile_override = id;
}
#endif
