// Host-side pieces shared by the operator files: context, error reporting, shape resolution.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "../../include/tilelink_mi355.h"
#include "tl_device.h"

struct tl_ctx {
  tl_config cfg;
  int device;
  int num_cus;
};

namespace tl {

void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);

#define TL_HIP(expr)                                                                          \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess) return tl::fail(TL_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// Tile shapes the GEMM kernels are instantiated for.
enum TileVariant { TILE_256x256 = 0, TILE_256x224 = 1, TILE_128x128 = 2, TILE_VARIANTS = 3 };

// Everything the host decides before a dense (AG+GEMM or GEMM+RS) launch.
struct Resolved {
  int variant, tile_m, tile_n;
  int nbm, nbn, n_tiles;
  int G, n_comm;
  int Tm_p, Tn_p;        // producer / reduce tile
  int n_ptm, n_ptn;      // producer or reduce tiles along rows / columns
  int rows_per_rank, rows_per_channel;
  int expected;          // producer tiles per channel (AG) ; not used by RS
  int threads, lds_bytes;
  int first_block;       // rotation of row blocks in the compute order
  int group_m;           // row blocks per group of the compute order
};

int resolve_dense(const tl_ctx* ctx, int op, int M, int N, int K, Resolved* r);

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

}  // namespace tl
